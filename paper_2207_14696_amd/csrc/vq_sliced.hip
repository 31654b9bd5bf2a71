// Vector-code decode with the codebooks in LDS (paper Sec. 3.2: each part's
// index selects one of `length` entries of `width` floats; Sec. 3.3 load, and
// the same fused with the neighbourhood mean of Appendix A.1).
//
// A decoded row is P lookups of width*4 bytes; served from L2 that is one
// request per 32..64 bytes, as many requests as the fp32 output itself.  The
// codebooks of all parts do not fit one CU's LDS (786 KB at 96 x 256 x 8), so
// the table's columns are sliced: a workgroup keeps the codebooks of SP
// consecutive parts (<= 64 KB) in LDS and produces only those SP*width output
// columns, for every requested row.  So that a slice does not have to pull a
// whole cache line out of a random packed row for its SP code bytes, a pre-pass
// first gathers the requested rows once (whole rows, 16 bytes per lane) and
// re-lays their codes slice-major into a scratch buffer, strips[s][i][SP]: each
// slice then streams its own strip.
//
// Lane mapping: LPS = SP*width/4 lanes cover one row's slice (4 output columns,
// one 16-byte LDS read and one 16-byte store each); a wave covers 64/LPS rows
// (gather_dequant) or destinations (gather_mean).
#include "common.hpp"

namespace bf {

namespace {

#ifndef BF_VQ_U
#define BF_VQ_U 4
#endif
constexpr int kVqThreads = 1024;  // 16 waves share one 64 KB codebook slice; two such groups per CU

struct VqGeom {
    int SP;    // parts per slice
    int NS;    // slices
    int LPS;   // lanes per row-slice
    bool ok;
};

VqGeom vq_geometry(const bifeat_params *p) {
    VqGeom g{0, 0, 0, false};
    const int w = p->scheme.vq_width, len = p->scheme.vq_length, P = p->P;
    if (w % 4 || (w & (w - 1)) || p->D % w) return g;  // 16-byte granules, whole parts
    int sp = 1;
    while (sp * 2 * len * w * 4 <= 65536 && sp * 2 * w / 4 <= 64 && sp * 2 <= 64) sp *= 2;
    while (sp > P) sp >>= 1;
    if (sp * len * w * 4 > 65536 || sp % 4) return g;  // slice's code bytes are whole dwords
    if ((int64_t)((P + sp - 1) / sp) * sp > p->rb) return g;  // strips copy whole slices of the padded row
    g.SP = sp;
    g.NS = (P + sp - 1) / sp;
    g.LPS = sp * w / 4;
    g.ok = true;
    return g;
}

__device__ inline void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// strips[s][i][0..SP) = codes[idx[i]][s*SP .. (s+1)*SP): a wave fetches 64/c16 whole
// rows (16 bytes per lane), parks them in LDS and writes them out slice-major, each
// slice's piece of the tile as one contiguous run.
__global__ __launch_bounds__(kThreads) void vq_strips_kernel(
    const uint4 *__restrict__ codes16, int c16, const int64_t *__restrict__ idx, int64_t M, int SP,
    int NS, uint32_t *__restrict__ strips) {
    __shared__ uint4 s_raw[kThreads];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint4 *raw = s_raw + wave * 64;
    const int RT = 64 / c16, r = lane / c16, c = lane - r * c16;
    const int SPW = SP >> 2, rbw = c16 * 4;  // dwords per slice piece / per row
    const int64_t tiles = (M + RT - 1) / RT;
    const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
    for (int64_t tile = (int64_t)blockIdx.x * (kThreads / 64) + wave; tile < tiles; tile += n_waves) {
        const int64_t row0 = tile * RT;
        const int nrow = (int)min((int64_t)RT, M - row0);
        if (r < nrow) raw[lane] = codes16[idx[row0 + r] * c16 + c];
        wave_sync();
        const uint32_t *raw32 = reinterpret_cast<const uint32_t *>(raw);
        const int per_slice = nrow * SPW, total = per_slice * NS;
        for (int u = lane; u < total; u += 64) {
            const int sl = u / per_slice, rem = u - sl * per_slice;
            const int rr = rem / SPW, k = rem - rr * SPW;
            strips[((int64_t)sl * M + row0) * SPW + rem] = raw32[rr * rbw + sl * SPW + k];
        }
        wave_sync();
    }
}

bool ensure_scratch(bifeat_params *p, size_t bytes) {
    if (p->scratch_bytes >= bytes) return true;
    if (p->d_scratch) (void)hipFree(p->d_scratch);  // waits for work that may still use it
    p->d_scratch = nullptr;
    p->scratch_bytes = 0;
    void *q = nullptr;
    if (hipMalloc(&q, bytes + bytes / 4) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    p->d_scratch = (uint8_t *)q;
    p->scratch_bytes = bytes + bytes / 4;
    return true;
}

void launch_strips(bifeat_params *p, const uint8_t *codes, const int64_t *idx, int64_t M,
                   const VqGeom &g, hipStream_t s) {
    const int c16 = (int)(p->rb / 16), RT = 64 / c16;
    const int64_t tiles = (M + RT - 1) / RT;
    int64_t blocks = (tiles + 3) / 4;
    if (blocks > (1 << 16)) blocks = 1 << 16;
    if (blocks < 1) blocks = 1;
    vq_strips_kernel<<<(unsigned)blocks, kThreads, 0, s>>>((const uint4 *)codes, c16, idx, M, g.SP,
                                                         g.NS, (uint32_t *)p->d_scratch);
}

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  All
// slices that walk the same rows are placed on one XCD (consecutive in its
// dispatch order), so that the packed rows they all re-read are fetched into
// that L2 once instead of once per XCD.
__device__ inline void slice_and_lane(int NS, int &slice, int &by, int &ny) {
    const int b = blockIdx.x, xcd = b & 7, j = b >> 3;
    slice = j % NS;
    by = (j / NS) * 8 + xcd;
    ny = gridDim.x / NS;  // multiple of 8
}

__device__ inline void load_slice(float *s_cb, const float *__restrict__ cb, int slice, int SP,
                                  int P, int len, int w) {
    const int parts = min(SP, P - slice * SP);
    const int n4 = parts * len * w / 4;
    const float4 *src = reinterpret_cast<const float4 *>(cb + (int64_t)slice * SP * len * w);
    float4 *dst = reinterpret_cast<float4 *>(s_cb);
    for (int i = threadIdx.x; i < n4; i += blockDim.x) dst[i] = src[i];
    __syncthreads();
}

// out[i, slice columns] = codebook entries selected by strip s of request i
__global__ __launch_bounds__(kVqThreads) void gather_dequant_vq_sliced_kernel(
    const uint32_t *__restrict__ strips, int64_t M, int D, int P, int w, int len, int SP, int NS,
    int lps_log2, const float *__restrict__ cb, float *__restrict__ out) {
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
    const int SPW = SP >> 2, word_off = pl >> 2, shift = 8 * (pl & 3);
    const uint32_t *strip = strips + (int64_t)slice * M * SPW + word_off;
    const float *entry0 = s_cb + (int64_t)pl * len * w + dim0;
    const int64_t tiles = (M + (1 << rpw_log2) - 1) >> rpw_log2;
    const int64_t stride = (int64_t)ny * nw;
    constexpr int U = BF_VQ_U;  // independent rows in flight per lane
    for (int64_t t0 = (int64_t)by * nw + wave; t0 < tiles; t0 += stride * U) {
        int64_t i[U];
        uint32_t word[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            i[u] = ((t0 + u * stride) << rpw_log2) + r_in;
            word[u] = (active && i[u] < M) ? strip[i[u] * SPW] : 0u;
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            if (active && i[u] < M) {
                const int c = (word[u] >> shift) & 0xFF;
                const float4 v = *reinterpret_cast<const float4 *>(entry0 + c * w);
                store_stream(reinterpret_cast<float4 *>(out + i[u] * D + col), v);
            }
        }
    }
}

// out[v, slice columns] = mean over the list of codebook entries
__global__ __launch_bounds__(kVqThreads) void gather_mean_vq_sliced_kernel(
    const uint32_t *__restrict__ strips, int64_t E, const int64_t *__restrict__ indptr, int64_t V,
    int D, int P, int w, int len, int SP, int NS, int lps_log2, const float *__restrict__ cb,
    float *__restrict__ out) {
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
    const int SPW = SP >> 2, word_off = pl >> 2, shift = 8 * (pl & 3);
    const uint32_t *strip = strips + (int64_t)slice * E * SPW + word_off;
    const float *entry0 = s_cb + (int64_t)pl * len * w + dim0;
    const int64_t tiles = (V + (1 << rpw_log2) - 1) >> rpw_log2;
    const int64_t stride = (int64_t)ny * nw;
    constexpr int U = BF_VQ_U;  // neighbours in flight per lane
    constexpr int kRun = 32;  // fp32 partial sums over runs of kRun, runs combined in fp64
    for (int64_t tile = (int64_t)by * nw + wave; tile < tiles; tile += stride) {
        const int64_t v = (tile << rpw_log2) + r_in;
        if (!active || v >= V) continue;
        const int64_t beg = indptr[v], end = indptr[v + 1];
        double total[4] = {0.0, 0.0, 0.0, 0.0};
        for (int64_t c0 = beg; c0 < end; c0 += kRun) {
            const int64_t c1 = min(end, c0 + kRun);
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
            for (int64_t e = c0; e < c1; e += U) {
                uint32_t word[U];
#pragma unroll
                for (int u = 0; u < U; u++) word[u] = strip[min(e + u, c1 - 1) * SPW];
#pragma unroll
                for (int u = 0; u < U; u++) {
                    const int c = (word[u] >> shift) & 0xFF;
                    const float4 q = *reinterpret_cast<const float4 *>(entry0 + c * w);
                    const float keep = e + u < c1 ? 1.0f : 0.0f;
                    acc[0] += keep * q.x;
                    acc[1] += keep * q.y;
                    acc[2] += keep * q.z;
                    acc[3] += keep * q.w;
                }
            }
#pragma unroll
            for (int k = 0; k < 4; k++) total[k] += (double)acc[k];
        }
        const double inv_n = end > beg ? 1.0 / (double)(end - beg) : 0.0;
        store_stream(reinterpret_cast<float4 *>(out + v * D + col),
                     make_float4((float)(total[0] * inv_n), (float)(total[1] * inv_n),
                                 (float)(total[2] * inv_n), (float)(total[3] * inv_n)));
    }
}

inline int ilog2(int x) {
    int l = 0;
    while ((1 << l) < x) l++;
    return l;
}

}  // namespace

// Both return false (nothing launched) when the codebook shape is outside what
// the sliced kernels handle (width not a power of two >= 4, D % 4 != 0, ...).
bool launch_gather_dequant_vq_sliced(bifeat_params *p, const uint8_t *codes, const int64_t *idx,
                                     int64_t M, float *out, hipStream_t s) {
    const VqGeom g = vq_geometry(p);
    if (!g.ok || (uintptr_t)out % 16 || p->rb / 16 > 64) return false;
    if (!ensure_scratch(p, (size_t)g.NS * M * g.SP)) return false;
    launch_strips(p, codes, idx, M, g, s);
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
    const int rpw = 64 / g.LPS;
    const int64_t tiles = (M + rpw - 1) / rpw;
    int64_t by = (tiles + (kVqThreads / 64) * 4 - 1) / ((kVqThreads / 64) * 4);
    const int64_t cap = (512 + g.NS - 1) / g.NS * 4;  // ~2 workgroups per CU, a few rounds
    if (by > cap) by = cap;
    by = (by + 7) / 8 * 8;
    const size_t shm = sizeof(float) * (size_t)g.SP * len * w;
    gather_dequant_vq_sliced_kernel<<<(unsigned)(g.NS * by), kVqThreads, shm, s>>>(
        (const uint32_t *)p->d_scratch, M, (int)p->D, p->P, w, len, g.SP, g.NS, ilog2(g.LPS),
        p->d_cb, out);
    return true;
}

bool launch_gather_mean_vq_sliced(bifeat_params *p, const uint8_t *codes, const int64_t *indptr,
                                  const int64_t *indices, int64_t V, int64_t E, float *out,
                                  hipStream_t s) {
    const VqGeom g = vq_geometry(p);
    if (!g.ok || (uintptr_t)out % 16 || p->rb / 16 > 64) return false;
    if (!ensure_scratch(p, (size_t)g.NS * (E > 0 ? E : 1) * g.SP)) return false;
    if (E > 0) launch_strips(p, codes, indices, E, g, s);
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
    const int rpw = 64 / g.LPS;
    const int64_t tiles = (V + rpw - 1) / rpw;
    int64_t by = (tiles + (kVqThreads / 64) - 1) / (kVqThreads / 64);
    const int64_t cap = (512 + g.NS - 1) / g.NS * 8;
    if (by > cap) by = cap;
    by = (by + 7) / 8 * 8;
    const size_t shm = sizeof(float) * (size_t)g.SP * len * w;
    gather_mean_vq_sliced_kernel<<<(unsigned)(g.NS * by), kVqThreads, shm, s>>>(
        (const uint32_t *)p->d_scratch, E, indptr, V, (int)p->D, p->P, w, len, g.SP, g.NS,
        ilog2(g.LPS), p->d_cb, out);
    return true;
}

}  // namespace bf
