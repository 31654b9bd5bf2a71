// Aggregation over fp32 rows: the layers after the first (Appendix A.1), where the
// neighbourhood mean runs over the previous layer's output instead of packed codes,
// and the row-length reduction of the scale profile (Appendix A.1, A.5).
//
// Both are row gathers bound by HBM: a row of D floats is fetched whole, 16 bytes per
// lane, several rows in flight per lane; nothing is staged.
#include "common.hpp"

namespace bf {
namespace {

constexpr int kAggInFlight = 4;  // rows in flight per lane
constexpr int kItemsPerGroup = 4;  // (destination, tile) items a lane group works through
// A list longer than kLong is not walked by one lane group (a hub's thousands of rows,
// one latency after the other, would outlast the rest of the launch): it is cut into
// pieces of kSub list entries that many groups sum side by side and add into the output
// row with atomics.  A workgroup of that kernel looks after kRange consecutive list
// entries, which at most kRange / kLong + 2 long lists can overlap.
constexpr int kLong = 256;
constexpr int kRange = 2048;
constexpr int kSub = 64;
constexpr int kMaxLong = kRange / kLong + 2;

// Compensated (Kahan) running sums: the rounding error of a sum stays at a couple of
// ulps of the mean magnitude whatever the list length; the kernel waits on memory, so
// the three extra operations per element cost nothing.  (Compiled without contraction
// or reassociation, which this relies on.)
__device__ inline void kahan_add(float &s, float &c, const float r) {
    const float y = r - c;
    const float t = s + y;
    c = (t - s) - y;
    s = t;
}

template <int VEC>
struct Acc;
template <>
struct Acc<4> {
    float4 v, c;
    __device__ void zero() { v = c = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ static float4 load(const float *p) { return *reinterpret_cast<const float4 *>(p); }
    __device__ void add(const float4 r) {
        kahan_add(v.x, c.x, r.x);
        kahan_add(v.y, c.y, r.y);
        kahan_add(v.z, c.z, r.z);
        kahan_add(v.w, c.w, r.w);
    }
    __device__ void store(float *p, int n, bool sum) const {
        float4 o = v;
        if (!sum) {
            const float d = (float)n;
            o = n > 0 ? make_float4(v.x / d, v.y / d, v.z / d, v.w / d) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        store_stream(reinterpret_cast<float4 *>(p), o);
    }
    // this piece's share of the row: partial sum (divided by the whole list's length)
    __device__ void add_to(float *p, int n, bool sum) const {
        const float d = (float)n;
        unsafeAtomicAdd(p + 0, sum ? v.x : v.x / d);
        unsafeAtomicAdd(p + 1, sum ? v.y : v.y / d);
        unsafeAtomicAdd(p + 2, sum ? v.z : v.z / d);
        unsafeAtomicAdd(p + 3, sum ? v.w : v.w / d);
    }
};
template <>
struct Acc<1> {
    float v, c;
    __device__ void zero() { v = c = 0.f; }
    __device__ static float load(const float *p) { return *p; }
    __device__ void add(const float r) { kahan_add(v, c, r); }
    __device__ void store(float *p, int n, bool sum) const {
        __builtin_nontemporal_store(sum ? v : (n > 0 ? v / (float)n : 0.f), p);
    }
    __device__ void add_to(float *p, int n, bool sum) const {
        unsafeAtomicAdd(p, sum ? v : v / (float)n);
    }
};

// rows of `pieces` consecutive list entries [e, end) added into acc, U loads in flight
template <int VEC, int U>
__device__ inline void add_rows(Acc<VEC> &acc, const float *__restrict__ base, int64_t D,
                                const int64_t *__restrict__ indices, int64_t e, int64_t end) {
    for (; e + U <= end; e += U) {
        decltype(Acc<VEC>::load(base)) r[U];
#pragma unroll
        for (int k = 0; k < U; k++) r[k] = Acc<VEC>::load(base + indices[e + k] * D);
#pragma unroll
        for (int k = 0; k < U; k++) acc.add(r[k]);
    }
    for (; e < end; e++) acc.add(Acc<VEC>::load(base + indices[e] * D));
}

// The lists of up to kLong entries.  A group of `lpr` lanes (a power of two up to 64)
// owns one (destination, column tile) item at a time: lane t of the group accumulates
// columns VEC*(tile*lpr + t) .. +VEC-1 over the destination's list, in list order
// (fp32, compensated).  Items are numbered tile-fastest so that neighbouring groups
// write one contiguous row.  Long lists are left to long_lists().
template <int VEC>
__device__ inline void short_lists(const float *__restrict__ x, int64_t D,
                                   const int64_t *__restrict__ indptr,
                                   const int64_t *__restrict__ indices, int64_t V, int lpr_log2,
                                   int tiles, int sum, float *__restrict__ out, int64_t block,
                                   int64_t nblocks) {
    const int lpr = 1 << lpr_log2;
    const int t = threadIdx.x & (lpr - 1);
    const int64_t groups = (nblocks * kThreads) >> lpr_log2;
    const int64_t items = V * tiles;
    for (int64_t item = (block * kThreads + threadIdx.x) >> lpr_log2; item < items; item += groups) {
        const int64_t v = item / tiles;
        const int tile = (int)(item - v * tiles);
        const int64_t col = (int64_t)VEC * (tile * lpr + t);
        const int64_t beg = indptr[v], end = indptr[v + 1];
        if (col >= D || end - beg > kLong) continue;
        Acc<VEC> acc;
        acc.zero();
        add_rows<VEC, kAggInFlight>(acc, x + col, D, indices, beg, end);
        acc.store(out + v * D + col, (int)(end - beg), sum != 0);
    }
}

// The long lists: a workgroup looks after kRange consecutive list entries at a time.  It
// finds the first destination whose list reaches into that range (a 64-way search in
// indptr by one wave), walks on from there, notes the long lists with the part that
// falls inside the range, and its lane groups sum pieces of kSub entries of those parts,
// each piece added to the output row, which aggregate_zero_long_kernel has zeroed.
template <int VEC>
__device__ inline void long_lists(const float *__restrict__ x, int64_t D,
                                  const int64_t *__restrict__ indptr,
                                  const int64_t *__restrict__ indices, int64_t V, int64_t E,
                                  int lpr_log2, int tiles, int sum, float *__restrict__ out,
                                  int64_t block, int64_t nblocks) {
    __shared__ int64_t s_v[kMaxLong], s_beg[kMaxLong], s_end[kMaxLong], s_first;
    __shared__ int s_deg[kMaxLong], s_n;
    const int lpr = 1 << lpr_log2;
    const int t = threadIdx.x & (lpr - 1);
    const int group = threadIdx.x >> lpr_log2, groups = kThreads >> lpr_log2;
    constexpr int kPieces = kRange / kSub;
    for (int64_t r0 = block * kRange; r0 < E; r0 += nblocks * kRange) {
        const int64_t r1 = r0 + kRange < E ? r0 + kRange : E;
        if (threadIdx.x < 64) {
            // first v with indptr[v + 1] > r0: 64 probes a round, evenly spaced over [lo, hi)
            int64_t lo = 0, hi = V;
            while (lo < hi) {
                const int64_t step = (hi - lo + 63) >> 6;
                const int64_t probe = lo + (int64_t)threadIdx.x * step;
                const uint64_t valid = __ballot(probe < hi);
                const uint64_t hit = __ballot(probe < hi && indptr[probe + 1] > r0);
                if (hit == 0) {
                    lo += (int64_t)(__popcll(valid) - 1) * step + 1;  // past the last probe
                } else {
                    const int j = __ffsll((unsigned long long)hit) - 1;
                    hi = lo + j * step;
                    if (j > 0) lo += (int64_t)(j - 1) * step + 1;
                }
            }
            if (threadIdx.x == 0) {
                s_first = lo;
                s_n = 0;
            }
        }
        __syncthreads();
        // walk the destinations from there until one starts at or after r1
        for (int64_t v0 = s_first;; v0 += kThreads) {
            const int64_t v = v0 + threadIdx.x;
            bool past = v >= V;
            if (!past) {
                const int64_t beg = indptr[v];
                past = beg >= r1;
                if (!past) {
                    const int64_t end = indptr[v + 1];
                    if (end - beg > kLong) {
                        const int k = atomicAdd(&s_n, 1);
                        if (k < kMaxLong) {
                            s_v[k] = v;
                            s_beg[k] = beg > r0 ? beg : r0;
                            s_end[k] = end < r1 ? end : r1;
                            s_deg[k] = (int)(end - beg);
                        }
                    }
                }
            }
            if (__syncthreads_or(past)) break;
        }
        const int n_long = s_n < kMaxLong ? s_n : kMaxLong;
        const int work = n_long * kPieces * tiles;
        for (int it = group; it < work; it += groups) {
            const int tile = it % tiles;
            const int piece = (it / tiles) % kPieces;
            const int k = it / (tiles * kPieces);
            const int64_t b = s_beg[k] + (int64_t)piece * kSub;
            const int64_t col = (int64_t)VEC * (tile * lpr + t);
            if (b >= s_end[k] || col >= D) continue;
            const int64_t end = b + kSub < s_end[k] ? b + kSub : s_end[k];
            Acc<VEC> acc;
            acc.zero();
            add_rows<VEC, 2 * kAggInFlight>(acc, x + col, D, indices, b, end);
            acc.add_to(out + s_v[k] * D + col, s_deg[k], sum != 0);
        }
        __syncthreads();
    }
}

// One launch for both: the first `long_blocks` workgroups (dispatched first; their
// pieces are the longest single chains of the launch) take the long lists, the rest
// the short ones.  The two write disjoint rows.
template <int VEC>
__global__ __launch_bounds__(kThreads) void aggregate_rows_kernel(
    const float *__restrict__ x, int64_t D, const int64_t *__restrict__ indptr,
    const int64_t *__restrict__ indices, int64_t V, int64_t E, int lpr_log2, int tiles, int sum,
    int long_blocks, float *__restrict__ out) {
    if ((int)blockIdx.x < long_blocks)
        long_lists<VEC>(x, D, indptr, indices, V, E, lpr_log2, tiles, sum, out, blockIdx.x,
                        long_blocks);
    else
        short_lists<VEC>(x, D, indptr, indices, V, lpr_log2, tiles, sum, out,
                         (int64_t)blockIdx.x - long_blocks, (int64_t)gridDim.x - long_blocks);
}

// Output rows of the long lists set to zero ahead of the launch above: a lane per
// destination looks at its list length, the wave then clears each long one's row.
__global__ __launch_bounds__(kThreads) void aggregate_zero_long_kernel(
    const int64_t *__restrict__ indptr, int64_t V, int64_t D, float *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    // whole waves stay in the loop together: the bound is rounded up to the wave
    for (int64_t v0 = (int64_t)blockIdx.x * kThreads + (threadIdx.x & ~63); v0 < V; v0 += stride) {
        const int64_t v = v0 + lane;
        const bool is_long = v < V && indptr[v + 1] - indptr[v] > kLong;
        uint64_t m = __ballot(is_long);
        while (m) {
            const int j = __ffsll((unsigned long long)m) - 1;
            m &= m - 1;
            float *row = out + (v0 + j) * D;
            for (int64_t c = lane; c < D; c += 64) row[c] = 0.f;
        }
    }
}

// acc[0] += sum over rows of sqrt(sum_j h[i][j]^2): one wave per row, squares and
// their sum in fp64, one atomic per workgroup.
template <int VEC>
__global__ __launch_bounds__(kThreads) void row_length_sum_kernel(const float *__restrict__ h,
                                                                  int64_t n, int64_t D,
                                                                  double *__restrict__ acc) {
    __shared__ double s_part[kThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t waves = (int64_t)gridDim.x * (kThreads / 64);
    double total = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * (kThreads / 64) + wave; i < n; i += waves) {
        const float *row = h + i * D;
        double q = 0.0;
        if constexpr (VEC == 4) {
            for (int64_t j = 4 * lane; j < D; j += 256) {
                const float4 r = *reinterpret_cast<const float4 *>(row + j);
                q += (double)r.x * r.x;
                q += (double)r.y * r.y;
                q += (double)r.z * r.z;
                q += (double)r.w * r.w;
            }
        } else {
            for (int64_t j = lane; j < D; j += 64) q += (double)row[j] * row[j];
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) q += __shfl_xor(q, m, 64);
        total += sqrt(q);
    }
    if (lane == 0) s_part[wave] = total;
    __syncthreads();
    if (threadIdx.x == 0) {
        double b = 0.0;
        for (int k = 0; k < kThreads / 64; k++) b += s_part[k];
        if (b != 0.0) atomicAdd(acc, b);
    }
}

bool vec_ok(const void *a, const void *b, int64_t D) {
    return D % 4 == 0 && (uintptr_t)a % 16 == 0 && (uintptr_t)b % 16 == 0;
}

}  // namespace

hipError_t launch_aggregate_rows(const float *x, int64_t D, const int64_t *indptr,
                                 const int64_t *indices, int64_t V, int64_t E, int sum, float *out,
                                 hipStream_t s) {
    const bool vec = vec_ok(x, out, D);
    const int64_t granules = vec ? D / 4 : D;
    int lpr_log2 = 2;  // at least four lanes per row
    while (lpr_log2 < 6 && ((int64_t)1 << lpr_log2) < granules) lpr_log2++;
    const int64_t tiles = (granules + ((int64_t)1 << lpr_log2) - 1) >> lpr_log2;
    const int64_t threads = (V * tiles) << lpr_log2;
    // many small workgroups rather than one resident set: the two kinds of work take turns
    // on the CUs as slots free up, and no workgroup's share is large enough to form a tail
    const int short_blocks = blocks_for((threads + kItemsPerGroup - 1) / kItemsPerGroup, 1 << 20);
    int long_blocks = 0;
    if (E > kLong) {  // otherwise no list is long
        const int64_t ranges = (E + kRange - 1) / kRange;
        long_blocks = (int)(ranges < (1 << 20) ? ranges : (1 << 20));
        aggregate_zero_long_kernel<<<blocks_for(V, 8 * 256), kThreads, 0, s>>>(indptr, V, D, out);
    }
    const int blocks = short_blocks + long_blocks;
    if (vec)
        aggregate_rows_kernel<4><<<blocks, kThreads, 0, s>>>(x, D, indptr, indices, V, E, lpr_log2,
                                                            (int)tiles, sum, long_blocks, out);
    else
        aggregate_rows_kernel<1><<<blocks, kThreads, 0, s>>>(x, D, indptr, indices, V, E, lpr_log2,
                                                            (int)tiles, sum, long_blocks, out);
    return hipGetLastError();
}

// a small fill kernel instead of a memset node: callers may capture the stream into a graph
__global__ void zero_doubles_kernel(double *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0;
}

void launch_zero_doubles(double *p, int n, hipStream_t s) {
    zero_doubles_kernel<<<(n + 127) / 128, 128, 0, s>>>(p, n);
}

hipError_t launch_row_length_sum(const float *h, int64_t n, int64_t D, double *acc, hipStream_t s) {
    const int blocks = blocks_for(n * 64, 8 * 256);
    if (vec_ok(h, h, D))
        row_length_sum_kernel<4><<<blocks, kThreads, 0, s>>>(h, n, D, acc);
    else
        row_length_sum_kernel<1><<<blocks, kThreads, 0, s>>>(h, n, D, acc);
    return hipGetLastError();
}

}  // namespace bf
