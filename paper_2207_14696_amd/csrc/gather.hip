// Per-iteration load (paper Sec. 3.3): gather the packed rows of the sampled
// nodes, and the fused gather + unpack + decode (Sec. 3.1 Eq. (2); Sec. 3.2
// codebook lookup).
//
// gather_dequant writes 4*D bytes per row and reads at most D bytes, so the
// mapping is output-centric: a lane owns 4 consecutive output columns (one
// 16-byte store, consecutive lanes consecutive addresses) and fetches only the
// 4*bits code bits it needs.  The lane keeps its column group for its whole
// life, so scale/offset sit in registers.
#include "common.hpp"

namespace bf {

// out[i, :] = codes[idx[i], :], 16 bytes per lane
__global__ __launch_bounds__(kThreads) void gather_codes_kernel(const uint4 *__restrict__ codes,
                                                               int rc /* 16B chunks per row */,
                                                               const int64_t *__restrict__ idx,
                                                               int64_t M, uint4 *__restrict__ out) {
    const uint32_t total = gridDim.x * kThreads;
    const uint32_t rows_per_pass = total / (uint32_t)rc;
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    if (t >= rows_per_pass * (uint32_t)rc) return;
    const int c = (int)(t % (uint32_t)rc);
    for (int64_t i = t / rc; i < M; i += rows_per_pass) store_stream(&out[i * rc + c], codes[idx[i] * rc + c]);
}

hipError_t launch_gather_codes(bifeat_params *p, const uint8_t *codes, const int64_t *idx,
                               int64_t M, uint8_t *out, hipStream_t s) {
    const int rc = (int)(p->rb / 16);
    int64_t want = M * rc;
    int blocks = blocks_for(want);
    if ((int64_t)blocks * kThreads < rc) blocks = (rc + kThreads - 1) / kThreads;
    gather_codes_kernel<<<blocks, kThreads, 0, s>>>((const uint4 *)codes, rc, idx, M, (uint4 *)out);
    return hipGetLastError();
}

// the 4*BITS code bits of columns 4g..4g+3 of a packed row (always inside the
// 16-byte padded row)
template <int BITS>
__device__ inline uint32_t code_bits4(const uint8_t *row, int g) {
    if constexpr (BITS == 8) return *reinterpret_cast<const uint32_t *>(row + 4 * g);
    else if constexpr (BITS == 4) return *reinterpret_cast<const uint16_t *>(row + 2 * g);
    else if constexpr (BITS == 2) return row[g];
    else return (uint32_t)(row[g >> 1] >> (4 * (g & 1))) & 0xFu;
}

template <bool VEC>
__device__ inline void store4(float *out, int64_t row, int D, int col0, const float v[4]) {
    float *dst = out + row * D + col0;
    if constexpr (VEC) {
        store_stream(reinterpret_cast<float4 *>(dst), make_float4(v[0], v[1], v[2], v[3]));
    } else {
#pragma unroll
        for (int k = 0; k < 4; k++)
            if (col0 + k < D) dst[k] = v[k];
    }
}

enum { DEC_UNIFORM = 0, DEC_LOG = 1 };

// scalar codes.  uniform: x' = fma(q, scale_j, min_j); log: x' = V[q] (table in LDS)
template <int BITS, int DEC, bool VEC>
__global__ __launch_bounds__(kThreads) void gather_dequant_sq_kernel(
    const uint8_t *__restrict__ codes, int64_t rb, const int64_t *__restrict__ idx, int64_t M,
    int D, const float *__restrict__ pa, const float *__restrict__ pb, float *__restrict__ out) {
    __shared__ float s_lut[DEC == DEC_LOG ? (1 << BITS) : 1];
    if constexpr (DEC == DEC_LOG) {
        for (int i = threadIdx.x; i < (1 << BITS); i += kThreads) s_lut[i] = pa[i];
        __syncthreads();
    }
    const int G = (D + 3) / 4;
    // grids stay below 2^20 workgroups: 32-bit thread ids and divisions
    const uint32_t total = gridDim.x * kThreads;
    const uint32_t rows_per_pass = total / (uint32_t)G;
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    if (t >= rows_per_pass * (uint32_t)G) return;
    const int g = (int)(t % (uint32_t)G), col0 = 4 * g;
    float mn[4], sc[4];
    if constexpr (DEC == DEC_UNIFORM) {
#pragma unroll
        for (int k = 0; k < 4; k++) {
            bool ok = col0 + k < D;
            mn[k] = ok ? pa[col0 + k] : 0.f;
            sc[k] = ok ? pb[col0 + k] : 0.f;
        }
    }
    constexpr uint32_t mask = (1u << BITS) - 1u;
#pragma unroll 4
    for (int64_t i = t / G; i < M; i += rows_per_pass) {
        const uint32_t bits = code_bits4<BITS>(codes + idx[i] * rb, g);
        float v[4];
#pragma unroll
        for (int k = 0; k < 4; k++) {
            uint32_t q = (bits >> (BITS * k)) & mask;
            if constexpr (DEC == DEC_UNIFORM) v[k] = fmaf((float)q, sc[k], mn[k]);
            else v[k] = s_lut[q];
        }
        store4<VEC>(out, i, D, col0, v);
    }
}

// Tile form of the scalar-code kernel (output rows 16-byte aligned, packed row
// of at most 64 16-byte chunks).  A wavefront takes RT = 64/c16 consecutive
// output rows: one 16-byte load per lane fetches their packed rows in whole
// sectors (sub-dword gathers cost an L2 request per few lanes), the raw codes
// are parked in LDS, and the tile's output span - contiguous in memory - is
// written with consecutive 16-byte stores, granule m of the span by lane m%64.
template <int BITS, int DEC>
__global__ __launch_bounds__(kThreads) void gather_dequant_tile_kernel(
    const uint4 *__restrict__ codes16, int c16, int s16, const int64_t *__restrict__ idx, int64_t M, int D,
    const float *__restrict__ pa, const float *__restrict__ pb, float *__restrict__ out) {
    extern __shared__ uint32_t smem[];
    constexpr int kLut = 1 << BITS;
    const int npar = DEC == DEC_UNIFORM ? 2 * D : kLut;  // D % 4 == 0 here
    float *s_par = reinterpret_cast<float *>(smem);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint4 *raw = reinterpret_cast<uint4 *>(smem + ((npar + 3) & ~3)) + wave * 64;
    for (int i = threadIdx.x; i < npar; i += kThreads) {
        if constexpr (DEC == DEC_UNIFORM) s_par[i] = i < D ? pb[i] : pa[i - D];  // [scale | min]
        else s_par[i] = pa[i];
    }
    __syncthreads();

    const int RT = 64 / c16;
    const int r = lane / c16, c = lane - r * c16;
    const int nf4 = D >> 2;
    const int step_d = 64 / nf4, step_f = 64 % nf4;
    const int lane_d = lane / nf4, lane_f = lane % nf4;
    const int rb = c16 * 16;
    const int64_t tiles = (M + RT - 1) / RT;
    const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
    constexpr uint32_t mask = (1u << BITS) - 1u;
    for (int64_t tile = (int64_t)blockIdx.x * (kThreads / 64) + wave; tile < tiles; tile += n_waves) {
        const int64_t row0 = tile * RT;
        const int nrow = (int)min((int64_t)RT, M - row0);
        if (r < nrow) raw[lane] = codes16[idx[row0 + r] * s16 + c];  // lane = r*c16 + c
        wave_sync();
        float4 *span = reinterpret_cast<float4 *>(out + row0 * D);
        const int ngran = nrow * nf4;
        int d = lane_d, f = lane_f;
#pragma unroll 2
        for (int m = lane; m < ngran; m += 64) {
            const uint8_t *rowp = reinterpret_cast<const uint8_t *>(raw) + d * rb;
            const uint32_t bits = code_bits4<BITS>(rowp, f);
            float4 v;
            if constexpr (DEC == DEC_UNIFORM) {
                const float4 a = *reinterpret_cast<const float4 *>(s_par + 4 * f);
                const float4 b = *reinterpret_cast<const float4 *>(s_par + D + 4 * f);
                v.x = fmaf((float)(bits & mask), a.x, b.x);
                v.y = fmaf((float)((bits >> BITS) & mask), a.y, b.y);
                v.z = fmaf((float)((bits >> (2 * BITS)) & mask), a.z, b.z);
                v.w = fmaf((float)((bits >> (3 * BITS)) & mask), a.w, b.w);
            } else {
                v.x = s_par[bits & mask];
                v.y = s_par[(bits >> BITS) & mask];
                v.z = s_par[(bits >> (2 * BITS)) & mask];
                v.w = s_par[(bits >> (3 * BITS)) & mask];
            }
            store_stream(&span[m], v);
            d += step_d;
            f += step_f;
            if (f >= nf4) {
                f -= nf4;
                d++;
            }
        }
        wave_sync();  // raw is rewritten by the next tile
    }
}

// input contract check (option "validate"): one pass over the indices and list bounds
__global__ void validate_zero_kernel(int32_t *bad) { *bad = 0; }

__global__ __launch_bounds__(kThreads) void validate_kernel(const int64_t *__restrict__ idx, int64_t M,
                                                           int64_t N,
                                                           const int64_t *__restrict__ indptr,
                                                           int64_t V, int64_t E, int64_t max_len,
                                                           int32_t *bad) {
    int wrong = 0;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < M; i += stride)
        wrong |= idx[i] < 0 || idx[i] >= N;
    if (indptr) {
        for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < V; v += stride)
            wrong |= indptr[v] > indptr[v + 1] || indptr[v] < 0 ||
                     (max_len > 0 && indptr[v + 1] - indptr[v] > max_len);
        if (blockIdx.x == 0 && threadIdx.x == 0) wrong |= indptr[0] != 0 || indptr[V] != E;
    }
    if (wrong) atomicOr(bad, 1);
}

void launch_validate(const int64_t *idx, int64_t M, int64_t N, const int64_t *indptr, int64_t V,
                     int64_t E, int64_t max_len, int32_t *d_bad, hipStream_t s) {
    validate_zero_kernel<<<1, 1, 0, s>>>(d_bad);
    const int64_t n = M > V ? M : V;
    validate_kernel<<<blocks_for(n > 0 ? n : 1), kThreads, 0, s>>>(idx, M, N, indptr, V, E, max_len, d_bad);
}

// vector codes: columns 4g..4g+3 of part p = col / w come from entry q = index p of
// the row (CB bytes per index)
template <int CB>
__device__ inline int vq_index(const uint8_t *row, int part) {
    if constexpr (CB == 1) return row[part];
    else return reinterpret_cast<const uint16_t *>(row)[part];
}

template <bool W4, int CB>
__global__ __launch_bounds__(kThreads) void gather_dequant_vq_kernel(
    const uint8_t *__restrict__ codes, int64_t rb, const int64_t *__restrict__ idx, int64_t M,
    int D, int w, int len, const float *__restrict__ cb, float *__restrict__ out) {
    const int G = (D + 3) / 4;
    // grids stay below 2^20 workgroups: 32-bit thread ids and divisions
    const uint32_t total = gridDim.x * kThreads;
    const uint32_t rows_per_pass = total / (uint32_t)G;
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    if (t >= rows_per_pass * (uint32_t)G) return;
    const int g = (int)(t % (uint32_t)G), col0 = 4 * g;
    int part[4], dim[4];
#pragma unroll
    for (int k = 0; k < 4; k++) {
        part[k] = (col0 + k) / w;
        dim[k] = (col0 + k) % w;
    }
#pragma unroll 2
    for (int64_t i = t / G; i < M; i += rows_per_pass) {
        const uint8_t *row = codes + idx[i] * rb;
        float v[4];
        if constexpr (W4) {  // w % 4 == 0: the four columns share a part, entry rows 16B aligned
            const int q = vq_index<CB>(row, part[0]);
            float4 c = *reinterpret_cast<const float4 *>(cb + ((int64_t)part[0] * len + q) * w + dim[0]);
            v[0] = c.x; v[1] = c.y; v[2] = c.z; v[3] = c.w;
        } else {
#pragma unroll
            for (int k = 0; k < 4; k++) {
                v[k] = 0.f;
                if (col0 + k < D) v[k] = cb[((int64_t)part[k] * len + vq_index<CB>(row, part[k])) * w + dim[k]];
            }
        }
        store4<W4>(out, i, D, col0, v);
    }
}

// Tile form for vector codes whose codebooks stay in L2 (width % 4 == 0, output
// rows 16-byte aligned): as gather_dequant_tile_kernel, a wavefront fetches the
// packed rows of RT = 64/c16 consecutive requests with one 16-byte load per lane
// and parks them in LDS; granule m of the tile's contiguous output span is then
// one 16-byte read of a codebook entry - kVqInFlight of them in flight per lane,
// the lanes of a part reading one contiguous entry - and one streaming store.
constexpr int kVqInFlight = 8;

template <int CB>
__global__ __launch_bounds__(kThreads) void gather_dequant_vq_tile_kernel(
    const uint4 *__restrict__ codes16, int c16, int s16, const int64_t *__restrict__ idx, int64_t M, int D,
    int w, int len, const float *__restrict__ cb, float *__restrict__ out) {
    __shared__ uint4 s_raw[kThreads];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint4 *raw = s_raw + wave * 64;
    const int RT = 64 / c16;
    const int r = lane / c16, c = lane - r * c16;
    const int nf4 = D >> 2;
    const int step_d = 64 / nf4, step_f = 64 % nf4;
    const int lane_d = lane / nf4, lane_f = lane % nf4;
    const int rb = c16 * 16;
    const int64_t tiles = (M + RT - 1) / RT;
    const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
    constexpr int U = kVqInFlight;
    for (int64_t tile = (int64_t)blockIdx.x * (kThreads / 64) + wave; tile < tiles; tile += n_waves) {
        const int64_t row0 = tile * RT;
        const int nrow = (int)min((int64_t)RT, M - row0);
        if (r < nrow) raw[lane] = codes16[idx[row0 + r] * s16 + c];  // lane = r*c16 + c
        wave_sync();
        float4 *span = reinterpret_cast<float4 *>(out + row0 * D);
        const int ngran = nrow * nf4;
        int d = lane_d, f = lane_f;
        for (int m0 = lane; m0 < ngran; m0 += 64 * U) {
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
                // granules past the tile's end re-read its last granule's entry (in bounds)
                const bool in = m0 + 64 * u < ngran;
                const int dd = in ? d : nrow - 1, ff = in ? f : nf4 - 1;
                const int col = 4 * ff, part = col / w, dim = col - part * w;
                const int q = vq_index<CB>(reinterpret_cast<const uint8_t *>(raw) + dd * rb, part);
                v[u] = *reinterpret_cast<const float4 *>(cb + ((int64_t)part * len + q) * w + dim);
                d += step_d;
                f += step_f;
                if (f >= nf4) {
                    f -= nf4;
                    d++;
                }
            }
#pragma unroll
            for (int u = 0; u < U; u++)
                if (m0 + 64 * u < ngran) store_stream(&span[m0 + 64 * u], v[u]);
        }
        wave_sync();  // raw is rewritten by the next tile
    }
}

hipError_t launch_gather_dequant(bifeat_params *p, const uint8_t *codes, const int64_t *idx,
                                 int64_t M, float *out, hipStream_t s, uint32_t *planes) {
    const int D = (int)p->D;
    const int G = (D + 3) / 4;
    const int vec = (D % 4 == 0) && ((uintptr_t)out % 16 == 0);
    int blocks = blocks_for((M * G + 3) / 4, p->opt_max_blocks > 0 ? p->opt_max_blocks : (1 << 20));
    if ((int64_t)blocks * kThreads < G) blocks = (G + kThreads - 1) / kThreads;
    const int kind = p->scheme.kind, bits = p->scheme.bits;
    if (kind == BIFEAT_VQ) {
        if (p->opt_vq_sliced && launch_gather_dequant_vq_sliced(p, codes, idx, M, out, s, planes))
            return hipGetLastError();
        const int w = p->scheme.vq_width;
        const int c16v = (int)(p->payload / 16), s16v = (int)(p->rb / 16);
        if (w % 4 == 0 && vec && c16v <= 64 && !p->opt_dequant_flat) {
            const int RT = 64 / c16v;
            const int64_t tiles = (M + RT - 1) / RT;
            const int64_t cap = p->opt_max_blocks > 0 ? p->opt_max_blocks : (1 << 16);
            const int64_t want = (tiles + 3) / 4;
            const int tb = (int)(want < cap ? want : cap);
            if (p->cbytes == 1)
                gather_dequant_vq_tile_kernel<1><<<tb, kThreads, 0, s>>>((const uint4 *)codes, c16v, s16v, idx, M, D, w, p->scheme.vq_length, p->d_cb, out);
            else
                gather_dequant_vq_tile_kernel<2><<<tb, kThreads, 0, s>>>((const uint4 *)codes, c16v, s16v, idx, M, D, w, p->scheme.vq_length, p->d_cb, out);
            return hipGetLastError();
        }
#define BF_GV(W4, CB) \
    gather_dequant_vq_kernel<W4, CB><<<blocks, kThreads, 0, s>>>(codes, p->rb, idx, M, D, w, p->scheme.vq_length, p->d_cb, out)
        if (w % 4 == 0 && vec) {
            if (p->cbytes == 1) BF_GV(true, 1);
            else BF_GV(true, 2);
        } else {
            if (p->cbytes == 1) BF_GV(false, 1);
            else BF_GV(false, 2);
        }
#undef BF_GV
        return hipGetLastError();
    }
    const int c16 = (int)(p->payload / 16), s16 = (int)(p->rb / 16);  // lanes per row / row stride
    // LDS of the tile kernel: the parameters (2*D floats for uniform codes) plus one 16-byte
    // slot per lane; tables too wide for the 64 KB a workgroup gets by default take the
    // flat kernel below
    const size_t tile_lds = sizeof(uint32_t) * (size_t)(((kind == BIFEAT_SQ_UNIFORM ? 2 * D : (1 << bits)) + 3) & ~3) +
                            (size_t)(kThreads / 64) * 64 * 16;
    if (vec && c16 <= 64 && !p->opt_dequant_flat && tile_lds <= 65536) {
        const int RT = 64 / c16;
        const int64_t tiles = (M + RT - 1) / RT;
        // about one tile per wave: the hardware's wave scheduling hides the index -> row ->
        // store latency better than a persistent, software-pipelined loop (measured); grids
        // beyond 2^16 workgroups lose again
        const int64_t cap = p->opt_max_blocks > 0 ? p->opt_max_blocks : (1 << 16);
        int64_t want = (tiles + 3) / 4;
        const int tb = (int)(want < cap ? want : cap);
        const size_t shm = tile_lds;
#define BF_GT(B, DEC, A, Bp) \
    gather_dequant_tile_kernel<B, DEC><<<tb, kThreads, shm, s>>>((const uint4 *)codes, c16, s16, idx, M, D, A, Bp, out)
        if (kind == BIFEAT_SQ_UNIFORM) {
            switch (bits) {
                case 1: BF_GT(1, DEC_UNIFORM, p->d_min, p->d_scale); break;
                case 2: BF_GT(2, DEC_UNIFORM, p->d_min, p->d_scale); break;
                case 4: BF_GT(4, DEC_UNIFORM, p->d_min, p->d_scale); break;
                default: BF_GT(8, DEC_UNIFORM, p->d_min, p->d_scale); break;
            }
        } else {
            switch (bits) {
                case 1: BF_GT(1, DEC_LOG, p->d_V, nullptr); break;
                case 2: BF_GT(2, DEC_LOG, p->d_V, nullptr); break;
                case 4: BF_GT(4, DEC_LOG, p->d_V, nullptr); break;
                default: BF_GT(8, DEC_LOG, p->d_V, nullptr); break;
            }
        }
#undef BF_GT
        return hipGetLastError();
    }
#define BF_GD(B, DEC, A, Bp)                                                                        \
    do {                                                                                                 \
        if (vec) gather_dequant_sq_kernel<B, DEC, true><<<blocks, kThreads, 0, s>>>(codes, p->rb, idx, M, D, A, Bp, out); \
        else gather_dequant_sq_kernel<B, DEC, false><<<blocks, kThreads, 0, s>>>(codes, p->rb, idx, M, D, A, Bp, out);    \
    } while (0)
    if (kind == BIFEAT_SQ_UNIFORM) {
        switch (bits) {
            case 1: BF_GD(1, DEC_UNIFORM, p->d_min, p->d_scale); break;
            case 2: BF_GD(2, DEC_UNIFORM, p->d_min, p->d_scale); break;
            case 4: BF_GD(4, DEC_UNIFORM, p->d_min, p->d_scale); break;
            default: BF_GD(8, DEC_UNIFORM, p->d_min, p->d_scale); break;
        }
    } else {
        switch (bits) {
            case 1: BF_GD(1, DEC_LOG, p->d_V, nullptr); break;
            case 2: BF_GD(2, DEC_LOG, p->d_V, nullptr); break;
            case 4: BF_GD(4, DEC_LOG, p->d_V, nullptr); break;
            default: BF_GD(8, DEC_LOG, p->d_V, nullptr); break;
        }
    }
#undef BF_GD
    return hipGetLastError();
}

}  // namespace bf
