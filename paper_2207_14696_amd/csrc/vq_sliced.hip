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
    int sp = 1;
    while (sp * 2 * len * w * 4 <= 65536 && sp * 2 * w / 4 <= 64 && sp * 2 <= 64) sp *= 2;
    while (sp > P) sp >>= 1;
    if (sp * len * w * 4 > 65536 || sp % 4) return g;  // slice's code bytes are whole dwords
    if ((int64_t)((P + sp - 1) / sp) * sp > p->rb) return g;  // strips copy whole slices of the padded row
    g.SP = sp;
    g.NS = (P + sp - 1) / sp;
    g.LPS = sp * w / 4;
    g.lds = sizeof(float) * (size_t)(len + 1) * sp * w;
    g.ok = true;
    return g;
}

__device__ inline void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Entries per strip: the request count plus slack, so that kernels may read a
// few entries past the end of a list (and mask them) and the pre-pass may write
// whole 16-byte chunks; a multiple of 16 keeps every strip 64-byte aligned.
inline int64_t strip_entries(int64_t M) { return (M + 8 + 15) / 16 * 16; }

constexpr int kStripK = 4;  // row batches per wave tile of the pre-pass

// strips[s][i][0..SP) = codes[idx[i]][s*SP .. (s+1)*SP), strip s starting at entry
// s*MS.  A wave fetches kStripK batches of 64/c16 whole rows (16 bytes per lane),
// parks them in LDS and writes each slice's piece of the tile as one contiguous
// run of 16-byte stores.
__global__ __launch_bounds__(kThreads) void vq_strips_kernel(
    const uint4 *__restrict__ codes16, int c16, const int64_t *__restrict__ idx, int64_t M, int SP,
    int NS, int64_t MS, uint32_t *__restrict__ strips) {
    constexpr int K = kStripK;
    __shared__ uint4 s_raw[(kThreads / 64) * K * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint4 *raw = s_raw + wave * (K * 64);
    const int RT = 64 / c16, r = lane / c16, c = lane - r * c16, TR = RT * K;
    const int SPW = SP >> 2, spw_log2 = __ffs(SPW) - 1, rbw = c16 * 4;  // dwords per slice piece / per row
    const int64_t tiles = (M + TR - 1) / TR;
    const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
    for (int64_t tile = (int64_t)blockIdx.x * (kThreads / 64) + wave; tile < tiles; tile += n_waves) {
        const int64_t row0 = tile * TR;
        const int nrow = (int)min((int64_t)TR, M - row0);
        uint4 v[K];
#pragma unroll
        for (int k = 0; k < K; k++) {
            const int rr = min(k * RT + r, nrow - 1);
            v[k] = codes16[idx[row0 + rr] * c16 + c];
        }
        if (r < RT) {
#pragma unroll
            for (int k = 0; k < K; k++) raw[(k * RT + r) * c16 + c] = v[k];
        }
        wave_sync();
        const uint32_t *raw32 = reinterpret_cast<const uint32_t *>(raw);
        const int chunks = (nrow * SPW + 3) >> 2, total = chunks * NS;
        for (int u = lane; u < total; u += 64) {
            const int sl = u / chunks, j = u - sl * chunks;
            uint32_t d[4];
#pragma unroll
            for (int t = 0; t < 4; t++) {
                const int lin = 4 * j + t, rr = min(lin >> spw_log2, TR - 1), k = lin & (SPW - 1);
                d[t] = raw32[rr * rbw + sl * SPW + k];
            }
            uint4 *dst = reinterpret_cast<uint4 *>(strips + ((int64_t)sl * MS + row0) * SPW) + j;
            *dst = make_uint4(d[0], d[1], d[2], d[3]);
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
    const int c16 = (int)(p->rb / 16), TR = (64 / c16) * kStripK;
    const int64_t tiles = (M + TR - 1) / TR;
    int64_t blocks = (tiles + 3) / 4;
    if (blocks > (1 << 16)) blocks = 1 << 16;
    if (blocks < 1) blocks = 1;
    vq_strips_kernel<<<(unsigned)blocks, kThreads, 0, s>>>((const uint4 *)codes, c16, idx, M, g.SP,
                                                         g.NS, strip_entries(M),
                                                         (uint32_t *)p->d_scratch);
}

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2; the
// slices that walk the same requests are placed on one XCD, consecutive in its
// dispatch order, so that what they all read (the list bounds) is fetched into
// that L2 once.
__device__ inline void slice_and_lane(int NS, int &slice, int &by, int &ny) {
    const int b = blockIdx.x, xcd = b & 7, j = b >> 3;
    slice = j % NS;
    by = (j / NS) * 8 + xcd;
    ny = gridDim.x / NS;  // multiple of 8
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
    const int w4 = w >> 2, per_part = len * w4, n4 = parts * per_part;
    const float4 *src = reinterpret_cast<const float4 *>(cb + (int64_t)slice * SP * len * w);
    float4 *dst = reinterpret_cast<float4 *>(s_cb);
    for (int i = threadIdx.x; i < n4; i += blockDim.x) {
        const int pl = i / per_part, rem = i - pl * per_part;
        const int c = rem / w4, k = rem - c * w4;
        dst[(c * SP + pl) * w4 + k] = src[i];
    }
    for (int i = threadIdx.x; i < SP * w4; i += blockDim.x)
        dst[len * SP * w4 + i] = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();
}

// out[i, slice columns] = codebook entries selected by strip s of request i
__global__ __launch_bounds__(kVqThreads) void gather_dequant_vq_sliced_kernel(
    const uint32_t *__restrict__ strips, int64_t M, int64_t MS, int D, int P, int w, int len, int SP,
    int NS, int lps_log2, const float *__restrict__ cb, float *__restrict__ out) {
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
    const uint32_t *strip = strips + (int64_t)slice * MS * SPW + word_off;
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
            word[u] = (active && i[u] < M) ? strip[i[u] * SPW] : 0u;
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            if (active && i[u] < M) {
                const int c = (word[u] >> shift) & 0xFF;
                const float4 v = *reinterpret_cast<const float4 *>(entry0 + c * cstride);
                store_stream(reinterpret_cast<float4 *>(out + i[u] * D + col), v);
            }
        }
    }
}

// out[v, slice columns] = mean over the list of codebook entries.  A lane owns
// CPL consecutive columns of one part (8 when the width allows: half the lanes,
// strip loads and address arithmetic per neighbour of the 4-column form - the
// kernel is bound by instruction issue, not by bytes).  The short form takes the
// lists of at most kRun neighbours - every list of a sampled block whose fan-out
// is that small - and sums and scales them in fp32; the long form takes the
// others, fp32 runs of kRun combined in fp64.  Each skips the other's lists.
constexpr int kRun = 32;

template <int CPL, bool LONG>
__global__ __launch_bounds__(kVqThreads) void gather_mean_vq_sliced_kernel(
    const uint8_t *__restrict__ strips, int64_t MS, const int64_t *__restrict__ indptr, int64_t V,
    int D, int P, int w, int len, int SP, int NS, int lps_log2, const float *__restrict__ cb,
    float *__restrict__ out) {
    extern __shared__ float s_cb[];
    int slice, by, ny;
    slice_and_lane(NS, slice, by, ny);
    load_slice(s_cb, cb, slice, SP, P, len, w);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int LPS = 1 << lps_log2, rpw_log2 = 6 - lps_log2;
    const int g = lane & (LPS - 1), r_in = lane >> lps_log2;
    const int pl = (CPL * g) / w, dim0 = (CPL * g) % w;
    const bool active = slice * SP + pl < P;
    const int col = (slice * SP + pl) * w + dim0;
    // byte offsets within the slice's strip fit 32 bits (checked by the launcher)
    const uint8_t *strip = strips + (int64_t)slice * MS * SP;
    const uint32_t lane_off = (uint32_t)(pl & ~3), shift = 8 * (pl & 3);
    const uint32_t cstride = (uint32_t)(SP * w) * 4u;  // bytes between entry rows in LDS
    const uint8_t *entry0 = reinterpret_cast<const uint8_t *>(s_cb + CPL * g);
    const uint32_t zero_row = (uint32_t)len;
    const int64_t tiles = (V + (1 << rpw_log2) - 1) >> rpw_log2;
    const int64_t stride = (int64_t)ny * nw;
    constexpr int U = BF_VQ_U;  // neighbours in flight per lane
    constexpr int Q = CPL / 4;

    // acc += entries selected by neighbours [e0, e1); reads up to U-1 strip entries past e1
    auto run = [&](uint32_t e0, uint32_t e1, float (&acc)[CPL]) {
        for (uint32_t e = e0; e < e1; e += U) {
            const uint32_t boff = e * (uint32_t)SP + lane_off;
            uint32_t word[U];
#pragma unroll
            for (int u = 0; u < U; u++)
                word[u] = *reinterpret_cast<const uint32_t *>(strip + (boff + (uint32_t)(u * SP)));
            float4 q[U][Q];
#pragma unroll
            for (int u = 0; u < U; u++) {
                uint32_t c = (word[u] >> shift) & 0xFFu;
                c = e + u < e1 ? c : zero_row;
                const uint8_t *ent = entry0 + c * cstride;
#pragma unroll
                for (int k = 0; k < Q; k++) q[u][k] = *reinterpret_cast<const float4 *>(ent + 16 * k);
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
#pragma unroll
                for (int k = 0; k < Q; k++) {
                    acc[4 * k + 0] += q[u][k].x;
                    acc[4 * k + 1] += q[u][k].y;
                    acc[4 * k + 2] += q[u][k].z;
                    acc[4 * k + 3] += q[u][k].w;
                }
            }
        }
    };

    for (int64_t tile = (int64_t)by * nw + wave; tile < tiles; tile += stride) {
        const int64_t v = (tile << rpw_log2) + r_in;
        if (!active || v >= V) continue;
        const int64_t beg = indptr[v], end = indptr[v + 1];
        const int64_t n = end - beg;
        if (LONG ? n <= kRun : n > kRun) continue;
        float res[CPL];
        if constexpr (!LONG) {
            float acc[CPL];
#pragma unroll
            for (int k = 0; k < CPL; k++) acc[k] = 0.0f;
            run((uint32_t)beg, (uint32_t)end, acc);
            const float inv_n = n > 0 ? 1.0f / (float)n : 0.0f;
#pragma unroll
            for (int k = 0; k < CPL; k++) res[k] = acc[k] * inv_n;
        } else {
            double total[CPL];
#pragma unroll
            for (int k = 0; k < CPL; k++) total[k] = 0.0;
            for (int64_t c0 = beg; c0 < end; c0 += kRun) {
                float acc[CPL];
#pragma unroll
                for (int k = 0; k < CPL; k++) acc[k] = 0.0f;
                run((uint32_t)c0, (uint32_t)min(end, c0 + kRun), acc);
#pragma unroll
                for (int k = 0; k < CPL; k++) total[k] += (double)acc[k];
            }
            const double inv_n = 1.0 / (double)n;
#pragma unroll
            for (int k = 0; k < CPL; k++) res[k] = (float)(total[k] * inv_n);
        }
#pragma unroll
        for (int k = 0; k < Q; k++)
            store_stream(reinterpret_cast<float4 *>(out + v * D + col + 4 * k),
                         make_float4(res[4 * k], res[4 * k + 1], res[4 * k + 2], res[4 * k + 3]));
    }
}

inline int ilog2(int x) {
    int l = 0;
    while ((1 << l) < x) l++;
    return l;
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

}  // namespace

// All return false (nothing launched) when the codebook shape is outside what
// the sliced kernels handle (width not a power of two >= 4, D % width != 0, ...).
bool launch_gather_dequant_vq_sliced(bifeat_params *p, const uint8_t *codes, const int64_t *idx,
                                     int64_t M, float *out, hipStream_t s) {
    const VqGeom g = vq_geometry(p);
    if (!g.ok || (uintptr_t)out % 16 || p->rb / 16 > 64) return false;
    if (!allow_lds(gather_dequant_vq_sliced_kernel, g.lds)) return false;
    const int64_t MS = strip_entries(M);
    if (!ensure_scratch(p, (size_t)g.NS * MS * g.SP)) return false;
    launch_strips(p, codes, idx, M, g, s);
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
    const int rpw = 64 / g.LPS;
    const int64_t tiles = (M + rpw - 1) / rpw;
    int64_t by = (tiles + (kVqThreads / 64) * 4 - 1) / ((kVqThreads / 64) * 4);
    const int64_t cap = (512 + g.NS - 1) / g.NS * 4;  // ~2 workgroups per CU, a few rounds
    if (by > cap) by = cap;
    by = (by + 7) / 8 * 8;
    gather_dequant_vq_sliced_kernel<<<(unsigned)(g.NS * by), kVqThreads, g.lds, s>>>(
        (const uint32_t *)p->d_scratch, M, MS, (int)p->D, p->P, w, len, g.SP, g.NS, ilog2(g.LPS),
        p->d_cb, out);
    return true;
}

// max_len: the caller's bound on the list lengths (0 = unknown); with a bound
// of at most kRun the long-list pass is not launched at all.
bool launch_gather_mean_vq_sliced(bifeat_params *p, const uint8_t *codes, const int64_t *indptr,
                                  const int64_t *indices, int64_t V, int64_t E, float *out,
                                  hipStream_t s) {
    const VqGeom g = vq_geometry(p);
    if (!g.ok || (uintptr_t)out % 16 || p->rb / 16 > 64) return false;
    const int64_t MS = strip_entries(E);
    if (MS * g.SP >= ((int64_t)1 << 32)) return false;  // 32-bit strip offsets
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
    const int cpl = w % 8 == 0 ? 8 : 4;  // columns per lane
    const bool with_long = !(p->opt_mean_max_degree > 0 && p->opt_mean_max_degree <= kRun);
#define BF_VQM(C, L) gather_mean_vq_sliced_kernel<C, L>
    if (cpl == 8 ? !(allow_lds(BF_VQM(8, false), g.lds) && allow_lds(BF_VQM(8, true), g.lds))
                 : !(allow_lds(BF_VQM(4, false), g.lds) && allow_lds(BF_VQM(4, true), g.lds)))
        return false;
    if (!ensure_scratch(p, (size_t)g.NS * MS * g.SP)) return false;
    if (E > 0) launch_strips(p, codes, indices, E, g, s);
    const int lps = g.LPS * 4 / cpl, rpw = 64 / lps;
    const int64_t tiles = (V + rpw - 1) / rpw;
    int64_t by = (tiles + (kVqThreads / 64) - 1) / (kVqThreads / 64);
    const int64_t cap = (512 + g.NS - 1) / g.NS * 8;
    if (by > cap) by = cap;
    by = (by + 7) / 8 * 8;
    const dim3 grid((unsigned)(g.NS * by));
#define BF_VQL(C, L)                                                                          \
    BF_VQM(C, L)<<<grid, kVqThreads, g.lds, s>>>(p->d_scratch, MS, indptr, V, (int)p->D, p->P, \
                                                 w, len, g.SP, g.NS, ilog2(lps), p->d_cb, out)
    if (cpl == 8) {
        BF_VQL(8, false);
        if (with_long) BF_VQL(8, true);
    } else {
        BF_VQL(4, false);
        if (with_long) BF_VQL(4, true);
    }
#undef BF_VQL
#undef BF_VQM
    return true;
}

}  // namespace bf
