// Vector-code decode with the codebooks in LDS (paper Sec. 3.2: each part's
// index selects one of `length` entries of `width` floats; Sec. 3.3 load, and
// the same fused with the neighbourhood mean of Appendix A.1).
//
// A decoded row is P lookups of width*4 bytes; served from L2 that is one
// request per 32..64 bytes, as many requests as the fp32 output itself.  The
// codebooks of all parts do not fit one CU's LDS (786 KB at 96 x 256 x 8), so
// the table's columns are sliced: a workgroup keeps the codebooks of SP
// consecutive parts (<= 64 KB) in LDS and produces only those SP*width output
// columns, for every requested row.  Different slices re-read the same packed
// rows (SP code bytes each); the rows are small and the slices walk the request
// list together, so those re-reads hit in L2.
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
    g.SP = sp;
    g.NS = (P + sp - 1) / sp;
    g.LPS = sp * w / 4;
    g.ok = true;
    return g;
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

// out[i, slice columns] = codebook entries of row idx[i]
__global__ __launch_bounds__(kVqThreads) void gather_dequant_vq_sliced_kernel(
    const uint8_t *__restrict__ codes, int64_t rb, const int64_t *__restrict__ idx, int64_t M,
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
    const int part = slice * SP + pl;
    const bool active = part < P;
    const int col = part * w + dim0;
    const int byte_off = part & ~3, shift = 8 * (part & 3);
    const float *entry0 = s_cb + (int64_t)pl * len * w + dim0;
    const int64_t tiles = (M + (1 << rpw_log2) - 1) >> rpw_log2;
    const int64_t stride = (int64_t)ny * nw;
    constexpr int U = BF_VQ_U;  // independent rows in flight per lane
    // row ids of the next iteration are requested one iteration ahead, so that each
    // iteration waits for one global round trip (the code words), not two
    int64_t row[U];
    const int64_t first = (int64_t)by * nw + wave;
#pragma unroll
    for (int u = 0; u < U; u++) {
        const int64_t i = ((first + u * stride) << rpw_log2) + r_in;
        row[u] = (active && i < M) ? idx[i] : 0;
    }
    for (int64_t t0 = first; t0 < tiles; t0 += stride * U) {
        int64_t i[U];
        uint32_t word[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            i[u] = ((t0 + u * stride) << rpw_log2) + r_in;
            const bool ok = active && i[u] < M;
            word[u] = ok ? *reinterpret_cast<const uint32_t *>(codes + row[u] * rb + byte_off) : 0u;
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int64_t in = ((t0 + (U + u) * stride) << rpw_log2) + r_in;
            row[u] = (active && in < M) ? idx[in] : 0;
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
    const uint8_t *__restrict__ codes, int64_t rb, const int64_t *__restrict__ indptr,
    const int64_t *__restrict__ indices, int64_t V, int D, int P, int w, int len, int SP,
    int NS, int lps_log2, const float *__restrict__ cb, float *__restrict__ out) {
    extern __shared__ float s_cb[];
    int slice, by, ny;
    slice_and_lane(NS, slice, by, ny);
    load_slice(s_cb, cb, slice, SP, P, len, w);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int LPS = 1 << lps_log2, rpw_log2 = 6 - lps_log2;
    const int g = lane & (LPS - 1), r_in = lane >> lps_log2;
    const int pl = (4 * g) / w, dim0 = (4 * g) % w;
    const int part = slice * SP + pl;
    const bool active = part < P;
    const int col = part * w + dim0;
    const int byte_off = part & ~3, shift = 8 * (part & 3);
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
                for (int u = 0; u < U; u++) {
                    const int64_t row = indices[min(e + u, c1 - 1)];
                    word[u] = *reinterpret_cast<const uint32_t *>(codes + row * rb + byte_off);
                }
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
    if (!g.ok || (uintptr_t)out % 16) return false;
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
    const int rpw = 64 / g.LPS;
    const int64_t tiles = (M + rpw - 1) / rpw;
    int64_t by = (tiles + (kVqThreads / 64) * 4 - 1) / ((kVqThreads / 64) * 4);
    const int64_t cap = (512 + g.NS - 1) / g.NS * 4;  // ~2 workgroups per CU, a few rounds
    if (by > cap) by = cap;
    by = (by + 7) / 8 * 8;
    const size_t shm = sizeof(float) * (size_t)g.SP * len * w;
    gather_dequant_vq_sliced_kernel<<<(unsigned)(g.NS * by), kVqThreads, shm, s>>>(
        codes, p->rb, idx, M, (int)p->D, p->P, w, len, g.SP, g.NS, ilog2(g.LPS), p->d_cb, out);
    return true;
}

bool launch_gather_mean_vq_sliced(bifeat_params *p, const uint8_t *codes, const int64_t *indptr,
                                  const int64_t *indices, int64_t V, float *out, hipStream_t s) {
    const VqGeom g = vq_geometry(p);
    if (!g.ok || (uintptr_t)out % 16) return false;
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
    const int rpw = 64 / g.LPS;
    const int64_t tiles = (V + rpw - 1) / rpw;
    int64_t by = (tiles + (kVqThreads / 64) - 1) / (kVqThreads / 64);
    const int64_t cap = (512 + g.NS - 1) / g.NS * 8;
    if (by > cap) by = cap;
    by = (by + 7) / 8 * 8;
    const size_t shm = sizeof(float) * (size_t)g.SP * len * w;
    gather_mean_vq_sliced_kernel<<<(unsigned)(g.NS * by), kVqThreads, shm, s>>>(
        codes, p->rb, indptr, indices, V, (int)p->D, p->P, w, len, g.SP, g.NS, ilog2(g.LPS), p->d_cb, out);
    return true;
}

}  // namespace bf
