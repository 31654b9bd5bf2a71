// Vector-code decode with the codebooks in LDS (paper Sec. 3.2: each part's
// index selects one of `length` entries of `width` floats; Sec. 3.3 load, and
// the same fused with the neighbourhood mean of Appendix A.1).
//
// A decoded row is P lookups of width*4 bytes; served from L2 that is one
// request per 32..64 bytes, as many requests as the fp32 output itself.  The
// codebooks of all parts do not fit one CU's LDS (786 KB at 96 x 256 x 8), so
// the table's columns are sliced: a workgroup keeps the codebooks of SP
// consecutive parts in LDS (as many as 64 KB hold, so that two workgroups share
// a CU; a single part of up to ~150 KB when one part alone is larger) and
// produces only those SP*width output columns, for every requested row.  So that a slice does not have to pull a
// whole cache line out of a random packed row for its SP code bytes, a pre-pass
// first gathers the requested rows once (whole rows, 16 bytes per lane) and
// writes them transposed at dword granularity into a scratch buffer,
// planes[k][i] = dword k of requested row i: the lane that decodes part p of
// consecutive requests then streams plane p/4.
//
// Lane mapping: LPS = SP*width/4 lanes cover one row's slice (4 output columns,
// one 16-byte LDS read and one 16-byte store each; gather_mean: 8 columns where
// the width allows); a wave covers 64/LPS rows (gather_dequant) or destinations
// (gather_mean).
#include <mutex>

#include "common.hpp"

namespace bf {

namespace {

#ifndef BF_VQ_U
#define BF_VQ_U 4
#endif
#ifndef BF_VQ_SUB
#define BF_VQ_SUB 4
#endif
constexpr int kVqThreads = 1024;  // 16 waves share one 64 KB codebook slice; two such groups per CU

struct VqGeom {
    int SP;      // parts per slice
    int NS;      // slices
    int LPS;     // 4-column lanes per row-slice
    size_t lds;  // bytes of LDS per workgroup: the slice's entries plus one all-zero entry row
    bool ok;
};

VqGeom vq_geometry(const bifeat_params *p) {
    VqGeom g{0, 0, 0, 0, false};
    const int w = p->scheme.vq_width, len = p->scheme.vq_length, P = p->P;
    if (w % 4 || (w & (w - 1)) || p->D % w) return g;  // 16-byte granules, whole parts
    const size_t part_bytes = sizeof(float) * (size_t)len * w;
    int sp = 1;
    if (part_bytes <= 65536) {
        // as many parts as 64 KB hold: two workgroups per CU
        while ((size_t)sp * 2 * part_bytes <= 65536 && sp * 2 * w / 4 <= 64 && sp * 2 <= 64) sp *= 2;
        while (sp > P) sp >>= 1;
    } else if (part_bytes + sizeof(float) * w > 156 * 1024) {
        return g;  // one part's codebook does not fit a CU's LDS
    }
    g.SP = sp;
    g.NS = (P + sp - 1) / sp;
    g.LPS = sp * w / 4;
    g.lds = sizeof(float) * (size_t)(len + 1) * sp * w;
    g.ok = true;
    return g;
}

// Entries per plane: the request count plus slack, so that kernels may read a
// few entries past the end of a list (and mask them) and the pre-pass may write
// whole 16-byte chunks; a multiple of 16 keeps every plane 64-byte aligned.
inline int64_t plane_entries(int64_t M) { return (M + 16 + 15) / 16 * 16; }

constexpr int kStripK = 4;  // row batches per wave tile of the pre-pass

// planes[k][i] = dword k of packed row idx[i], k < NPW, plane k starting at dword
// k*MS.  A wave fetches kStripK batches of 64/c16 whole rows (16 bytes per lane),
// parks them in LDS and writes each plane's piece of the tile as one contiguous
// run of 16-byte stores.
template <typename IT>
__global__ __launch_bounds__(kThreads) void vq_planes_kernel(
    const uint4 *__restrict__ codes16, int c16, int s16, const IT *__restrict__ idx, int64_t M, int NPW,
    int64_t MS, uint32_t *__restrict__ planes) {
    constexpr int K = kStripK;
    __shared__ uint4 s_raw[(kThreads / 64) * K * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint4 *raw = s_raw + wave * (K * 64);
    const int RT = 64 / c16, r = lane / c16, c = lane - r * c16, TR = RT * K;
    const int rbw = c16 * 4;  // dwords per packed row
    const int64_t tiles = (M + TR - 1) / TR;
    const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
    for (int64_t tile = (int64_t)blockIdx.x * (kThreads / 64) + wave; tile < tiles; tile += n_waves) {
        const int64_t row0 = tile * TR;
        const int nrow = (int)min((int64_t)TR, M - row0);
        uint4 v[K];
#pragma unroll
        for (int k = 0; k < K; k++) {
            const int rr = min(k * RT + r, nrow - 1);
            v[k] = codes16[(int64_t)idx[row0 + rr] * s16 + c];
        }
        if (r < RT) {
#pragma unroll
            for (int k = 0; k < K; k++) raw[(k * RT + r) * c16 + c] = v[k];
        }
        wave_sync();
        const uint32_t *raw32 = reinterpret_cast<const uint32_t *>(raw);
        const int chunks = (nrow + 3) >> 2, total = chunks * NPW;
        for (int u = lane; u < total; u += 64) {
            const int pk = u / chunks, j = u - pk * chunks;
            uint32_t d[4];
#pragma unroll
            for (int t = 0; t < 4; t++) d[t] = raw32[min(4 * j + t, TR - 1) * rbw + pk];
            uint4 *dst = reinterpret_cast<uint4 *>(planes + (int64_t)pk * MS + row0) + j;
            *dst = make_uint4(d[0], d[1], d[2], d[3]);
        }
        wave_sync();
    }
}

void launch_planes(bifeat_params *p, const uint8_t *codes, const void *idx, bool idx32, int64_t M,
                   uint32_t *planes, hipStream_t s) {
    const int c16 = (int)(p->payload / 16), s16 = (int)(p->rb / 16), TR = (64 / c16) * kStripK;
    const int64_t tiles = (M + TR - 1) / TR;
    int64_t blocks = (tiles + 3) / 4;
    if (blocks > (1 << 16)) blocks = 1 << 16;
    if (blocks < 1) blocks = 1;
    if (idx32)
        vq_planes_kernel<int32_t><<<(unsigned)blocks, kThreads, 0, s>>>(
            (const uint4 *)codes, c16, s16, (const int32_t *)idx, M, (int)(p->payload / 4), plane_entries(M), planes);
    else
        vq_planes_kernel<int64_t><<<(unsigned)blocks, kThreads, 0, s>>>(
            (const uint4 *)codes, c16, s16, (const int64_t *)idx, M, (int)(p->payload / 4), plane_entries(M), planes);
}

// workgroup b serves slice b % NS as that slice's (b / NS)-th of ny workgroups
__device__ inline void slice_and_lane(int NS, int &slice, int &by, int &ny) {
    const int b = blockIdx.x;
    slice = b % NS;
    by = b / NS;
    ny = ((int)gridDim.x - slice + NS - 1) / NS;
}

// LDS layout of a slice: s_cb[c][SP*w] - for each code value c the entries c of
// all SP parts side by side, so the lane that owns slice columns [x, x+4) reads
// 16 bytes at float offset c*SP*w + x.  Lanes that are served together own
// consecutive x, hence distinct banks whatever their codes are (the part-major
// layout of the global codebooks would make random codes collide).  Row `len`
// is all zeros: the entry a masked-out neighbour selects.
__device__ inline void load_slice(float *s_cb, const float *__restrict__ cb, int slice, int SP,
                                  int P, int len, int w) {
    const int parts = min(SP, P - slice * SP);
    const int w4 = w >> 2, w4_log2 = __ffs(w4) - 1, per_part = len * w4;
    const float4 *src = reinterpret_cast<const float4 *>(cb + (int64_t)slice * SP * len * w);
    float4 *dst = reinterpret_cast<float4 *>(s_cb);
    // thread -> (part, 16-byte piece) without integer division: groups of
    // `lanes` consecutive threads walk one part
    int lanes = 1;
    while (lanes * 2 <= (int)blockDim.x / SP) lanes *= 2;  // SP <= 64 < blockDim.x
    const int lanes_log2 = __ffs(lanes) - 1;
    const int pl = threadIdx.x >> lanes_log2, t = threadIdx.x & (lanes - 1);
    if (pl < parts) {
        for (int i = t; i < per_part; i += lanes) {
            const int c = i >> w4_log2, k = i & (w4 - 1);
            dst[(c * SP + pl) * w4 + k] = src[pl * per_part + i];
        }
    }
    for (int i = threadIdx.x; i < SP * w4; i += blockDim.x)
        dst[len * SP * w4 + i] = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();
}

// out[i, slice columns] = codebook entries selected by the planes of request i
__global__ __launch_bounds__(kVqThreads) void gather_dequant_vq_sliced_kernel(
    const uint32_t *__restrict__ planes, int64_t M, int64_t MS, int D, int P, int w, int len, int SP,
    int NS, int lps_log2, int cbytes, const float *__restrict__ cb, float *__restrict__ out) {
    extern __shared__ float s_cb[];
    int slice, by, ny;
    slice_and_lane(NS, slice, by, ny);
    load_slice(s_cb, cb, slice, SP, P, len, w);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int LPS = 1 << lps_log2, rpw_log2 = 6 - lps_log2;
    const int g = lane & (LPS - 1), r_in = lane >> lps_log2;
    const int pl = (4 * g) / w, dim0 = (4 * g) % w;
    const bool active = slice * SP + pl < P;
    const int col = (slice * SP + pl) * w + dim0;
    // the part's index: cbytes bytes at byte (part * cbytes) of the packed row
    const int boff = (slice * SP + pl) * cbytes, shift = 8 * (boff & 3);
    const uint32_t cmask = cbytes == 1 ? 0xFFu : 0xFFFFu;
    const uint32_t *plane = planes + (int64_t)(boff >> 2) * MS;
    const float *entry0 = s_cb + 4 * g;
    const int cstride = SP * w;
    const int64_t tiles = (M + (1 << rpw_log2) - 1) >> rpw_log2;
    const int64_t stride = (int64_t)ny * nw;
    constexpr int U = BF_VQ_U;  // independent rows in flight per lane
    for (int64_t t0 = (int64_t)by * nw + wave; t0 < tiles; t0 += stride * U) {
        int64_t i[U];
        uint32_t word[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            i[u] = ((t0 + u * stride) << rpw_log2) + r_in;
            word[u] = (active && i[u] < M) ? plane[i[u]] : 0u;
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            if (active && i[u] < M) {
                const int c = (int)((word[u] >> shift) & cmask);
                const float4 v = *reinterpret_cast<const float4 *>(entry0 + c * cstride);
                store_stream(reinterpret_cast<float4 *>(out + i[u] * D + col), v);
            }
        }
    }
}

// out[v, slice columns] = mean over the list of codebook entries.  A lane owns
// CPL consecutive columns of one part (8 when the width allows: half the lanes,
// plane loads and address arithmetic per neighbour of the 4-column form) and
// fetches the codes of four consecutive neighbours with one 16-byte load from
// its plane.  Two kernels share the work: the short one takes the lists of at
// most kRun neighbours - every list of a sampled block whose fan-out is that
// small - and sums and scales them in fp32; the long one takes the others, fp32
// runs of kRun combined in fp64.  Each skips the other's lists.
constexpr int kRun = 32;

struct __attribute__((aligned(4))) Words4 {
    uint32_t w[4];
};

// per-lane constants of the mean kernels
template <int CPL>
struct MeanLane {
    int slice, by, ny, lane, wave, nw, rpw_log2, g, r_in, col, cs_log2;
    bool active;
    const uint8_t *base, *lds;
    uint32_t plane_off, shift, cmask, entry0, zero_row;

    __device__ MeanLane(const uint32_t *planes, int64_t MS, const float *s_cb, int P, int w, int len,
                        int SP, int NS, int lps_log2, int cbytes) {
        slice_and_lane(NS, slice, by, ny);
        lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
        rpw_log2 = 6 - lps_log2;
        g = lane & ((1 << lps_log2) - 1), r_in = lane >> lps_log2;
        const int pl = (CPL * g) / w, dim0 = (CPL * g) % w;
        active = slice * SP + pl < P;
        col = (slice * SP + pl) * w + dim0;
        // byte offsets into the planes fit 32 bits (checked by the launcher)
        base = reinterpret_cast<const uint8_t *>(planes);
        // the part's index: cbytes bytes at byte (part * cbytes) of the packed row
        const int boff = (slice * SP + pl) * cbytes;
        // (lanes past the table's last part read plane 0: they fetch codes like the others and
        // drop them, and a plane of their own part number need not exist)
        plane_off = active ? (uint32_t)((boff >> 2) * MS) : 0u, shift = 8 * (boff & 3);
        cmask = cbytes == 1 ? 0xFFu : 0xFFFFu;
        cs_log2 = __ffs(SP * w * 4) - 1;  // log2 of the bytes between entry rows in LDS
        lds = reinterpret_cast<const uint8_t *>(s_cb);
        entry0 = (uint32_t)(CPL * g * 4);
        zero_row = (uint32_t)len;
    }

    // codes of neighbours e..e+3 (may run up to 3 entries past a list's end)
    __device__ Words4 words(uint32_t e) const {
        return *reinterpret_cast<const Words4 *>(base + ((plane_off + e) << 2));
    }

    // acc += the entries selected by the first min(rem, 4) codes of t, rem >= 1;
    // BF_VQ_SUB neighbours' LDS reads in flight at a time
    __device__ void add4(const Words4 &t, uint32_t rem, float (&acc)[CPL]) const {
        constexpr int Q = CPL / 4;
#pragma unroll
        for (int h = 0; h < 4; h += BF_VQ_SUB) {
            float4 q[BF_VQ_SUB][Q];
#pragma unroll
            for (int u = 0; u < BF_VQ_SUB; u++) {
                uint32_t c = (t.w[h + u] >> shift) & cmask;
                if (h + u > 0) c = (uint32_t)(h + u) < rem ? c : zero_row;
                const uint8_t *ent = lds + ((c << cs_log2) + entry0);
#pragma unroll
                for (int k = 0; k < Q; k++) q[u][k] = *reinterpret_cast<const float4 *>(ent + 16 * k);
            }
#pragma unroll
            for (int u = 0; u < BF_VQ_SUB; u++) {
#pragma unroll
                for (int k = 0; k < Q; k++) {
                    acc[4 * k + 0] += q[u][k].x;
                    acc[4 * k + 1] += q[u][k].y;
                    acc[4 * k + 2] += q[u][k].z;
                    acc[4 * k + 3] += q[u][k].w;
                }
            }
            if (BF_VQ_SUB < 4) asm volatile("" ::: "memory");
        }
    }

    // acc += entries selected by neighbours [e0, e1)
    __device__ void run(uint32_t e0, uint32_t e1, float (&acc)[CPL]) const {
        for (uint32_t e = e0; e < e1; e += 4) {
            Words4 t = words(e);
            // all four words in registers before the first is used (keeps the
            // compiler from splitting the load into per-neighbour branches)
            asm volatile("" : "+v"(t.w[0]), "+v"(t.w[1]), "+v"(t.w[2]), "+v"(t.w[3]));
            add4(t, e1 - e, acc);
        }
    }

    __device__ void store(float *__restrict__ out, int64_t v, int D, const float (&res)[CPL]) const {
#pragma unroll
        for (int k = 0; k < CPL / 4; k++)
            store_stream(reinterpret_cast<float4 *>(out + v * D + col + 4 * k),
                         make_float4(res[4 * k], res[4 * k + 1], res[4 * k + 2], res[4 * k + 3]));
    }

    // The same for a whole wave tile of 8-column lanes, without holes.  A lane's 32 bytes
    // are two 16-byte halves; stored half by half, each store instruction would write
    // every other 16 bytes of the tile's rows - a pattern that streaming stores drain at half
    // speed.  Instead the two halves of the wave trade: lanes 32..63 hand their first half to
    // lanes 0..31 in exchange for those lanes' second half (one cross-half swap per register),
    // so that the first instruction writes both halves of the destinations owned by lanes
    // 0..31 and the second both halves of the others: whole 128-byte lines per instruction.
    // `write`: this lane's destination is to be written; v: its destination.
    __device__ void store_tile(float *__restrict__ out, int64_t v, int D, const float (&res)[CPL],
                               bool write) const {
        static_assert(CPL == 8, "two 16-byte halves per lane");
        const unsigned long long wmask = __ballot(write);
        uint32_t a[4], b[4];
#pragma unroll
        for (int k = 0; k < 4; k++) {
            // a: [first halves of lanes 0..31 | second halves of lanes 0..31]
            // b: [first halves of lanes 32..63 | second halves of lanes 32..63]
            const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(res[k]), __float_as_uint(res[4 + k]),
                                                            false, false);
            a[k] = r[0];
            b[k] = r[1];
        }
        const bool upper = lane >= 32;
        const int64_t half_dst = 32 >> (6 - rpw_log2);  // destinations owned by half a wave
        // first instruction: destinations of lanes 0..31 (upper lanes write their partner's second half)
        const int64_t v0 = upper ? v - half_dst : v;
        const bool w0 = (wmask >> (lane & 31)) & 1ull;
        // second instruction: destinations of lanes 32..63 (lower lanes write their partner's first half)
        const int64_t v1 = upper ? v : v + half_dst;
        const bool w1 = (wmask >> (32 + (lane & 31))) & 1ull;
        const int c0 = col + (upper ? 4 : 0);
#ifdef BF_VQ_PLAIN
        if (w0) *reinterpret_cast<uint4 *>(out + v0 * D + c0) = make_uint4(a[0], a[1], a[2], a[3]);
        if (w1) *reinterpret_cast<uint4 *>(out + v1 * D + c0) = make_uint4(b[0], b[1], b[2], b[3]);
        return;
#endif
        if (w0)
            store_stream(reinterpret_cast<float4 *>(out + v0 * D + c0),
                         make_float4(__uint_as_float(a[0]), __uint_as_float(a[1]), __uint_as_float(a[2]),
                                     __uint_as_float(a[3])));
        if (w1)
            store_stream(reinterpret_cast<float4 *>(out + v1 * D + c0),
                         make_float4(__uint_as_float(b[0]), __uint_as_float(b[1]), __uint_as_float(b[2]),
                                     __uint_as_float(b[3])));
    }
};

// Short lists.  On this hardware a wave's loads return in issue order with its
// stores, so a load issued after a tile's output stores would wait for them to
// drain to memory.  The loop is therefore pipelined by hand: the list bounds of
// the tile after next and the first kPre*4 codes of the next tile are requested
// before the current tile's stores are issued, and are waited for only after.
#ifndef BF_VQ_PRE
#define BF_VQ_PRE 3
#endif
constexpr int kPre = BF_VQ_PRE;

template <int CPL>
__global__ __launch_bounds__(kVqThreads) void gather_mean_vq_short_kernel(
    const uint32_t *__restrict__ planes, int64_t MS, const int64_t *__restrict__ indptr, int64_t V,
    int D, int P, int w, int len, int SP, int NS, int lps_log2, int cbytes, int agg_sum,
    const float *__restrict__ cb, float *__restrict__ out, int alone, int32_t *__restrict__ status) {
    extern __shared__ float s_cb[];
    const MeanLane<CPL> L(planes, MS, s_cb, P, w, len, SP, NS, lps_log2, cbytes);
    load_slice(s_cb, cb, L.slice, SP, P, len, w);
    const int64_t tiles = (V + (1 << L.rpw_log2) - 1) >> L.rpw_log2;
    const int64_t stride = (int64_t)L.ny * L.nw;
    using Pair = HIP_vector_type<long long, 2>;
    // list bounds of the destination this lane serves in `tile` (clamped: always a valid address)
    auto bounds = [&](int64_t tile) {
        const int64_t v = min((tile << L.rpw_log2) + L.r_in, V - 1);
        return *reinterpret_cast<const Pair *>(indptr + v);
    };
    int64_t tile = (int64_t)L.by * L.nw + L.wave;
    if (tile >= tiles) return;
    Pair ip = bounds(tile);
    uint32_t beg = (uint32_t)ip.x, n = (uint32_t)(ip.y - ip.x);
    Words4 cur[kPre];
#pragma unroll
    for (int k = 0; k < kPre; k++) cur[k] = L.words(beg + 4 * k);
    Pair ip_next = bounds(tile + stride);
    for (; tile < tiles; tile += stride) {
        // requests for the tiles ahead, all issued before this tile's stores
        const uint32_t beg1 = (uint32_t)ip_next.x, n1 = (uint32_t)(ip_next.y - ip_next.x);
        Words4 nxt[kPre];
#pragma unroll
        for (int k = 0; k < kPre; k++) nxt[k] = L.words(beg1 + 4 * k);
        ip_next = bounds(tile + 2 * stride);
        asm volatile("" ::: "memory");

        const int64_t v = (tile << L.rpw_log2) + L.r_in;
        const bool mine = L.active && v < V && n <= (uint32_t)kRun;
        // no long-list pass follows when the caller promised short lists: a longer list gets a
        // row of NaNs instead of stale memory, and the handle's status word is raised
        const bool over = alone && L.active && v < V && !mine;
        float res[CPL];
#pragma unroll
        for (int k = 0; k < CPL; k++) res[k] = __builtin_nanf("");
        if (mine) {
            float acc[CPL];
#pragma unroll
            for (int k = 0; k < CPL; k++) acc[k] = 0.0f;
#pragma unroll
            for (int k = 0; k < kPre; k++)
                if ((uint32_t)(4 * k) < n) L.add4(cur[k], n - 4 * k, acc);
            if (n > 4 * kPre) L.run(beg + 4 * kPre, beg + n, acc);
            // 1 ulp reciprocal: far inside the 1e-5 budget
            const float inv_n = agg_sum ? 1.0f : (n > 0 ? __builtin_amdgcn_rcpf((float)n) : 0.0f);
#pragma unroll
            for (int k = 0; k < CPL; k++) res[k] = acc[k] * inv_n;
        }
        if (over && L.g == 0 && L.slice == 0) raise_status(status, kStatusListTooLong);
        if constexpr (CPL == 8) {
            L.store_tile(out, v, D, res, mine || over);
        } else {
            if (mine || over) L.store(out, v, D, res);
        }
        asm volatile("" ::: "memory");
        beg = beg1, n = n1;
#pragma unroll
        for (int k = 0; k < kPre; k++) cur[k] = nxt[k];
    }
}

template <int CPL>
__global__ __launch_bounds__(kVqThreads) void gather_mean_vq_long_kernel(
    const uint32_t *__restrict__ planes, int64_t MS, const int64_t *__restrict__ indptr, int64_t V,
    int D, int P, int w, int len, int SP, int NS, int lps_log2, int cbytes, int agg_sum,
    const float *__restrict__ cb, float *__restrict__ out) {
    extern __shared__ float s_cb[];
    const MeanLane<CPL> L(planes, MS, s_cb, P, w, len, SP, NS, lps_log2, cbytes);
    load_slice(s_cb, cb, L.slice, SP, P, len, w);
    const int64_t tiles = (V + (1 << L.rpw_log2) - 1) >> L.rpw_log2;
    const int64_t stride = (int64_t)L.ny * L.nw;
    for (int64_t tile = (int64_t)L.by * L.nw + L.wave; tile < tiles; tile += stride) {
        const int64_t v = (tile << L.rpw_log2) + L.r_in;
        if (!L.active || v >= V) continue;
        const int64_t beg = indptr[v], end = indptr[v + 1];
        if (end - beg <= kRun) continue;
        double total[CPL];
#pragma unroll
        for (int k = 0; k < CPL; k++) total[k] = 0.0;
        for (int64_t c0 = beg; c0 < end; c0 += kRun) {
            float acc[CPL];
#pragma unroll
            for (int k = 0; k < CPL; k++) acc[k] = 0.0f;
            L.run((uint32_t)c0, (uint32_t)min(end, c0 + kRun), acc);
#pragma unroll
            for (int k = 0; k < CPL; k++) total[k] += (double)acc[k];
        }
        const double inv_n = agg_sum ? 1.0 : 1.0 / (double)(end - beg);
        float res[CPL];
#pragma unroll
        for (int k = 0; k < CPL; k++) res[k] = (float)(total[k] * inv_n);
        L.store(out, v, D, res);
    }
}

// Two rounds of the mean (Appendix A.1 applied twice, nothing in between) for vector codes:
// planes hold the transposed codes of the outer block's list entries, in list order, so the
// outer list of seed-list entry u is the run [indptr1[u], indptr1[u+1]) of every plane.  A lane
// group owns a seed's slice columns: per entry it sums the selected codebook entries of that
// run (fp32 runs of kRun combined in fp64), divides by the run's length, and adds up in fp64.
// The chain seed list -> outer list's bounds -> codes is taken off the critical path: the
// group's lanes fetch the bounds of as many entries as the group has lanes at once and hand
// them round by lane exchange, and an entry's first kPre*4 codes are requested while the
// entry before it is summed.
template <int CPL>
__global__ __launch_bounds__(kVqThreads) void gather_mean_vq_2hop_kernel(
    const uint32_t *__restrict__ planes, int64_t MS, const int64_t *__restrict__ indptr1,
    const int64_t *__restrict__ indptr2, const int64_t *__restrict__ indices2, int64_t V2, int D,
    int P, int w, int len, int SP, int NS, int lps_log2, int cbytes, const float *__restrict__ cb,
    float *__restrict__ out) {
    extern __shared__ float s_cb[];
    const MeanLane<CPL> L(planes, MS, s_cb, P, w, len, SP, NS, lps_log2, cbytes);
    load_slice(s_cb, cb, L.slice, SP, P, len, w);
    const int64_t tiles = (V2 + (1 << L.rpw_log2) - 1) >> L.rpw_log2;
    const int64_t stride = (int64_t)L.ny * L.nw;
    const int lps = 1 << lps_log2;
    const int first_lane = L.lane & ~(lps - 1);  // lane 0 of this lane's group
    for (int64_t tile = (int64_t)L.by * L.nw + L.wave; tile < tiles; tile += stride) {
        const int64_t v = (tile << L.rpw_log2) + L.r_in;
        if (v >= V2) continue;  // whole groups leave together
        const int64_t beg2 = indptr2[v], end2 = indptr2[v + 1];
        double outer[CPL];
#pragma unroll
        for (int k = 0; k < CPL; k++) outer[k] = 0.0;
        for (int64_t e0 = beg2; e0 < end2; e0 += lps) {
            // bounds of the next `lps` entries, one per lane of the group
            uint32_t my_beg = 0u, my_n = 0u;
            if (e0 + L.g < end2) {
                const int64_t u = indices2[e0 + L.g];
                const int64_t b1 = indptr1[u];
                my_beg = (uint32_t)b1;
                my_n = (uint32_t)(indptr1[u + 1] - b1);
            }
            const int cnt = (int)min((int64_t)lps, end2 - e0);
            uint32_t beg = __shfl(my_beg, first_lane), n = __shfl(my_n, first_lane);
            Words4 cur[kPre];
#pragma unroll
            for (int k = 0; k < kPre; k++) cur[k] = L.words(beg + 4 * k);
            for (int j = 0; j < cnt; j++) {
                const int jn = min(j + 1, cnt - 1);
                const uint32_t beg1 = __shfl(my_beg, first_lane + jn), n1 = __shfl(my_n, first_lane + jn);
                Words4 nxt[kPre];
#pragma unroll
                for (int k = 0; k < kPre; k++) nxt[k] = L.words(beg1 + 4 * k);
                if (L.active && n > 0) {
                    const double inv1 = 1.0 / (double)n;
                    float acc[CPL];
#pragma unroll
                    for (int k = 0; k < CPL; k++) acc[k] = 0.0f;
                    if (n <= (uint32_t)kRun) {
#pragma unroll
                        for (int k = 0; k < kPre; k++)
                            if ((uint32_t)(4 * k) < n) L.add4(cur[k], n - 4 * k, acc);
                        if (n > 4 * kPre) L.run(beg + 4 * kPre, beg + n, acc);
#pragma unroll
                        for (int k = 0; k < CPL; k++) outer[k] += (double)acc[k] * inv1;
                    } else {
                        double total[CPL];
#pragma unroll
                        for (int k = 0; k < CPL; k++) total[k] = 0.0;
                        for (uint32_t c0 = beg; c0 < beg + n; c0 += kRun) {
#pragma unroll
                            for (int k = 0; k < CPL; k++) acc[k] = 0.0f;
                            L.run(c0, min(beg + n, c0 + (uint32_t)kRun), acc);
#pragma unroll
                            for (int k = 0; k < CPL; k++) total[k] += (double)acc[k];
                        }
#pragma unroll
                        for (int k = 0; k < CPL; k++) outer[k] += total[k] * inv1;
                    }
                }
                beg = beg1, n = n1;
#pragma unroll
                for (int k = 0; k < kPre; k++) cur[k] = nxt[k];
            }
        }
        if (L.active) {
            const double inv2 = end2 > beg2 ? 1.0 / (double)(end2 - beg2) : 0.0;
            float res[CPL];
#pragma unroll
            for (int k = 0; k < CPL; k++) res[k] = (float)(outer[k] * inv2);
            L.store(out, v, D, res);
        }
    }
}

// The slice plus its zero row can exceed the 64 KB a workgroup gets by default.
template <typename Kern>
bool allow_lds(Kern kern, size_t bytes) {
    if (bytes <= 65536) return true;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return true;
}

// workgroups: two fit a CU (LDS, registers); a few per slot so that the last
// ones to finish leave little of the chip idle, each loading its slice once
// (workgroup b serves slice b % NS: never fewer workgroups than slices)
int sliced_grid(const bifeat_params *p, int64_t wave_tiles, int64_t dflt, int NS) {
    int64_t blocks = (wave_tiles + (kVqThreads / 64) - 1) / (kVqThreads / 64);
    const int64_t cap = p->opt_max_blocks > 0 ? p->opt_max_blocks : dflt;
    if (blocks > cap) blocks = cap;
    if (blocks < NS) blocks = NS;
    return (int)blocks;
}

}  // namespace

// ---- the fixed workspace of bifeat_gather_dequant_static: one array per GPU, part of the
// library's code object (every GPU the library runs on holds it until the process ends).
// `scratch` is only a host-side stand-in for the symbol: the address kernels can use is
// looked up once per device and kept.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
uint8_t *g_static_ptr[kMaxDevices] = {};
}  // namespace

size_t static_scratch_bytes() { return kStaticScratchBytes; }

// The current device's copy of the array (hipSuccess and *out set, or the HIP error).
hipError_t static_scratch_ptr(uint8_t **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_static_ptr[dev] = (uint8_t *)ptr;
    }
    *out = g_static_ptr[dev];
    return hipSuccess;
}

size_t vq_gather_scratch_bytes(const bifeat_params *p, int64_t M) {
    return (size_t)p->payload * (size_t)plane_entries(M);
}

// All return false (nothing launched) when the codebook shape is outside what
// the sliced kernels handle (width not a power of two >= 4, D % width != 0, ...).
// planes: the workspace for the transposed codes (vq_gather_scratch_bytes(p, M) bytes), or
// nullptr for the handle's own, grown as needed.
bool launch_gather_dequant_vq_sliced(bifeat_params *p, const uint8_t *codes, const int64_t *idx,
                                     int64_t M, float *out, hipStream_t s, uint32_t *planes) {
    const VqGeom g = vq_geometry(p);
    if (!g.ok || (uintptr_t)out % 16 || p->payload / 16 > 64) return false;
    // a slice narrower than 256 bytes of output per row makes the stores too fine-grained
    // (measured: slower than decoding from L2 with whole rows per wave)
    if (g.LPS < 16) return false;
    if (!allow_lds(gather_dequant_vq_sliced_kernel, g.lds)) return false;
    const int64_t MS = plane_entries(M);
    if (!planes) {
        if (!ensure_scratch(p, (size_t)p->payload * MS, s)) return false;
        planes = (uint32_t *)p->d_scratch;
    }
    launch_planes(p, codes, idx, false, M, planes, s);
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
    const int rpw = 64 / g.LPS;
    const int64_t tiles = (M + rpw - 1) / rpw;
    const int grid = sliced_grid(p, (tiles + BF_VQ_U - 1) / BF_VQ_U * g.NS, 2048, g.NS);
    gather_dequant_vq_sliced_kernel<<<grid, kVqThreads, g.lds, s>>>(
        planes, M, MS, (int)p->D, p->P, w, len, g.SP, g.NS, ilog2(g.LPS),
        p->cbytes, p->d_cb, out);
    return true;
}

// With the caller's bound on the list lengths at most kRun, the long-list pass is not
// launched at all (a longer list then gets a row of NaNs and raises the status word).
bool launch_gather_mean_vq_sliced(bifeat_params *p, const MeanCall &c) {
    const VqGeom g = vq_geometry(p);
    if (!g.ok || (uintptr_t)c.out % 16 || p->payload / 16 > 64) return false;
    const int64_t MS = plane_entries(c.E);
    if (p->payload * MS >= ((int64_t)1 << 32)) return false;  // 32-bit plane offsets
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
    const int cpl = w % 8 == 0 ? 8 : 4;  // columns per lane
    const bool with_long = !(c.max_degree > 0 && c.max_degree <= kRun);
    if (cpl == 8 ? !(allow_lds(gather_mean_vq_short_kernel<8>, g.lds) &&
                     allow_lds(gather_mean_vq_long_kernel<8>, g.lds))
                 : !(allow_lds(gather_mean_vq_short_kernel<4>, g.lds) &&
                     allow_lds(gather_mean_vq_long_kernel<4>, g.lds)))
        return false;
    if (!ensure_scratch(p, (size_t)p->payload * MS, c.s)) return false;
    if (c.E > 0) launch_planes(p, c.codes, c.indices, c.idx32, c.E, (uint32_t *)p->d_scratch, c.s);
    const int lps = g.LPS * 4 / cpl, rpw = 64 / lps;
    const int64_t tiles = (c.V + rpw - 1) / rpw;
    const int grid = sliced_grid(p, tiles * g.NS, 1024, g.NS);
#define BF_VQA                                                                                  \
    (const uint32_t *)p->d_scratch, MS, c.indptr, c.V, (int)p->D, p->P, w, len, g.SP, g.NS,     \
        ilog2(lps), p->cbytes, c.agg_sum, p->d_cb, c.out
    if (cpl == 8) {
        gather_mean_vq_short_kernel<8><<<grid, kVqThreads, g.lds, c.s>>>(BF_VQA, with_long ? 0 : 1, c.status);
        if (with_long) gather_mean_vq_long_kernel<8><<<grid, kVqThreads, g.lds, c.s>>>(BF_VQA);
    } else {
        gather_mean_vq_short_kernel<4><<<grid, kVqThreads, g.lds, c.s>>>(BF_VQA, with_long ? 0 : 1, c.status);
        if (with_long) gather_mean_vq_long_kernel<4><<<grid, kVqThreads, g.lds, c.s>>>(BF_VQA);
    }
#undef BF_VQA
    return true;
}

// Two rounds in one call for vector codes with the codebooks in LDS: the pre-pass transposes
// the codes of the outer block's list entries, then one kernel walks seed lists over runs of
// the planes.  Any list length.  False (nothing launched) outside the sliced kernels' shapes or
// when the workspace cannot be had.
bool launch_gather_mean_2hop_vq_sliced(bifeat_params *p, const HopCall &c) {
    const VqGeom g = vq_geometry(p);
    if (!g.ok || (uintptr_t)c.out % 16 || p->payload / 16 > 64) return false;
    const int64_t MS = plane_entries(c.E1);
    if (p->payload * MS >= ((int64_t)1 << 32)) return false;  // 32-bit plane offsets
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
    const int cpl = w % 8 == 0 ? 8 : 4;
    if (cpl == 8 ? !allow_lds(gather_mean_vq_2hop_kernel<8>, g.lds) : !allow_lds(gather_mean_vq_2hop_kernel<4>, g.lds))
        return false;
    if (!ensure_scratch(p, (size_t)p->payload * MS, c.s)) return false;
    if (c.E1 > 0) launch_planes(p, c.codes, c.indices1, false, c.E1, (uint32_t *)p->d_scratch, c.s);
    const int lps = g.LPS * 4 / cpl, rpw = 64 / lps;
    const int64_t tiles = (c.V2 + rpw - 1) / rpw;
    const int grid = sliced_grid(p, tiles * g.NS, 1024, g.NS);
#define BF_VQH                                                                                   \
    (const uint32_t *)p->d_scratch, MS, c.indptr1, c.indptr2, c.indices2, c.V2, (int)p->D, p->P, w, \
        len, g.SP, g.NS, ilog2(lps), p->cbytes, p->d_cb, c.out
    if (cpl == 8) gather_mean_vq_2hop_kernel<8><<<grid, kVqThreads, g.lds, c.s>>>(BF_VQH);
    else gather_mean_vq_2hop_kernel<4><<<grid, kVqThreads, g.lds, c.s>>>(BF_VQH);
#undef BF_VQH
    return true;
}

}  // namespace bf
