// The streaming kernels of the one-time preprocessing (paper Sec. 3.3; code definitions
// Sec. 3.1 Eq. (1)), written against a *row source* instead of a pointer: the per-column
// range fit, the fit of the extreme magnitudes, and encode + pack of the scalar codes.
//
// A row source hands out the table's values; it is either a chunk resident in memory
// (ChunkSrc, what bifeat_fit_update / bifeat_quantize take) or a producer that makes the
// values on the fly (anything with the same three members, instantiated by the caller's
// own translation unit through include/bifeat_produce.hpp) - then the raw table never
// exists in memory at all, neither for the fit nor for the encoder (Appendix D: the
// preprocessing cost is one pass to fit and one to encode).
//
//   struct Src {
//       struct Ctx;                                        // per-thread state of a column group
//       __device__ void prepare(Ctx &, int col0, int D) const;   // once per thread
//       __device__ float4 load4(const Ctx &, int64_t r, int col0) const;  // columns col0..col0+3 of row r
//       __device__ float load1(const Ctx &, int64_t r, int col) const;    // one column of row r
//   };
//
// In all kernels a thread owns a fixed group of consecutive columns for its whole life (the
// grid's row stride is a multiple of the groups per row), so per-column parameters live in
// registers while consecutive lanes still touch consecutive addresses.
#pragma once

#include "common.hpp"

namespace bf {

// rows of a chunk in memory, row-major, element type T (float or __half)
template <typename T>
struct ChunkSrc {
    const T *x;
    int D;
    struct Ctx {};
    __device__ void prepare(Ctx &, int, int) const {}
    __device__ float4 load4(const Ctx &, int64_t r, int col0) const { return bf::load4(x + r * D + col0); }
    __device__ float load1(const Ctx &, int64_t r, int col) const { return bf::load1(x + r * D + col); }
};

// per-column min / max of the rows [0, rows) of `src` merged into the running state.
// VEC = 4 needs D % 4 == 0 (and, for a chunk in memory, 16-byte / 8-byte alignment).
template <class Src, int VEC>
__global__ __launch_bounds__(kThreads) void fit_minmax_kernel(Src src, int64_t rows, int D, int G,
                                                             int32_t *state, int use_lds) {
    extern __shared__ int32_t lds[];
    if (use_lds) {
        for (int i = threadIdx.x; i < D; i += kThreads) {
            lds[i] = kKeyPosInf;
            lds[D + i] = kKeyNegInf;
        }
        __syncthreads();
    }
    // A workgroup streams one contiguous piece of the chunk: kThreads/G whole rows per
    // iteration when a row's G column groups fit a workgroup (a wave's lanes then read
    // consecutive 16 bytes), else groups of G threads across the grid walk consecutive rows.
    const bool by_block = G <= kThreads;
    const int rpi = by_block ? kThreads / G : 0;  // rows per iteration of a workgroup
    const uint32_t total = gridDim.x * kThreads;
    const uint32_t rows_per_pass = total / (uint32_t)G;
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    const bool active = by_block ? (int)threadIdx.x < rpi * G : t < rows_per_pass * (uint32_t)G;
    if (active) {
        const int g = by_block ? (int)threadIdx.x % G : (int)(t % (uint32_t)G);
        float mn[VEC], mx[VEC];
#pragma unroll
        for (int k = 0; k < VEC; k++) {
            mn[k] = INFINITY;
            mx[k] = -INFINITY;
        }
        typename Src::Ctx ctx;
        src.prepare(ctx, g * VEC, D);
        int64_t rbeg, rend, rstep;
        if (by_block) {
            const int64_t per_block = (rows + gridDim.x - 1) / gridDim.x;
            rbeg = (int64_t)blockIdx.x * per_block + (int)threadIdx.x / G;
            rend = min(rows, (int64_t)(blockIdx.x + 1) * per_block);
            rstep = rpi;
        } else {
            const int64_t K = (rows + rows_per_pass - 1) / rows_per_pass;
            rbeg = (int64_t)(t / G) * K;
            rend = min(rows, rbeg + K);
            rstep = 1;
        }
#pragma unroll 4
        for (int64_t r = rbeg; r < rend; r += rstep) {
            float v[VEC];
            if constexpr (VEC == 4) {
                float4 q = src.load4(ctx, r, g * VEC);
                v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
            } else {
                v[0] = src.load1(ctx, r, g);
            }
#pragma unroll
            for (int k = 0; k < VEC; k++) {
                if (v[k] < mn[k]) mn[k] = v[k];  // NaN compares false: skipped
                if (v[k] > mx[k]) mx[k] = v[k];
            }
        }
        int32_t *lo = use_lds ? lds : state;
#pragma unroll
        for (int k = 0; k < VEC; k++) {
            int col = g * VEC + k;
            atomicMin(&lo[col], float_key(mn[k]));
            atomicMax(&lo[D + col], float_key(mx[k]));
        }
    }
    if (use_lds) {
        __syncthreads();
        // thousands of workgroups would hammer the same 2*D words: only those that improve
        // on the value already there (read without ordering: a stale read merely costs one
        // atomic that changes nothing) issue the atomic
        for (int i = threadIdx.x; i < D; i += kThreads) {
            const int32_t lo_k = lds[i], hi_k = lds[D + i];
            if (lo_k < __builtin_nontemporal_load(&state[i])) atomicMin(&state[i], lo_k);
            if (hi_k > __builtin_nontemporal_load(&state[D + i])) atomicMax(&state[D + i], hi_k);
        }
    }
}

// smallest nonzero and largest finite magnitude of the rows [0, rows) of a row source (log
// scheme); positive floats order like their bit patterns.  Thread = one group of VEC columns,
// rows interleaved across the grid.
template <class Src, int VEC>
__global__ __launch_bounds__(kThreads) void fit_log_rows_kernel(Src src, int64_t rows, int D, int G,
                                                               int32_t *state) {
    uint32_t mmin = 0x7F800000u, mmax = 0u;
    auto take = [&](float v) {
        const uint32_t m = __float_as_uint(fabsf(v));
        if (m < 0x7F800000u) {  // finite
            if (m != 0u && m < mmin) mmin = m;
            if (m > mmax) mmax = m;
        }
    };
    const uint32_t total = gridDim.x * kThreads;
    const uint32_t rows_per_pass = total / (uint32_t)G;
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    if (t < rows_per_pass * (uint32_t)G) {
        const int g = (int)(t % (uint32_t)G);
        typename Src::Ctx ctx;
        src.prepare(ctx, g * VEC, D);
#pragma unroll 4
        for (int64_t r = t / G; r < rows; r += rows_per_pass) {
            if constexpr (VEC == 4) {
                const float4 v = src.load4(ctx, r, g * VEC);
                take(v.x);
                take(v.y);
                take(v.z);
                take(v.w);
            } else {
                take(src.load1(ctx, r, g));
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        mmin = min(mmin, (uint32_t)__shfl_xor((int)mmin, o));
        mmax = max(mmax, (uint32_t)__shfl_xor((int)mmax, o));
    }
    if ((threadIdx.x & 63) == 0) {
        atomicMin((uint32_t *)&state[0], mmin);
        atomicMax((uint32_t *)&state[1], mmax);
    }
}

// ------------------------------------------------------------ scalar encoders
struct UniformCoder {
    static constexpr bool kEdges = false;
    const float *mn, *inv;
    float L;
    struct Ctx { float mn[4], inv[4]; };
    __device__ void prepare(Ctx &c, int col0, int D) const {
#pragma unroll
        for (int k = 0; k < 4; k++) {
            bool ok = col0 + k < D;
            c.mn[k] = ok ? mn[col0 + k] : 0.0f;
            c.inv[k] = ok ? inv[col0 + k] : 0.0f;
        }
    }
    // q = clamp(rne((x - min) * inv), 0, L); sub, mul, round are separate fp32
    // operations; max/min discard NaN, so NaN -> 0
    __device__ uint32_t code(const Ctx &c, float x, int k) const {
        float d = __fsub_rn(x, c.mn[k]);
        float t = __fmul_rn(d, c.inv[k]);
        float r = rintf(t);
        r = fminf(fmaxf(r, 0.0f), L);
        return (uint32_t)(int)r;
    }
};

struct LogCoder {
    static constexpr bool kEdges = true;
    const float *T;  // global, H-1 edges
    int H;
    struct Ctx { const float *edges; };
    __device__ void prepare(Ctx &c, int, int) const { c.edges = nullptr; }
    // l = #{i : |x| >= T_i} by bisection over the sorted edges (in LDS)
    __device__ uint32_t code(const Ctx &c, float x, int) const {
        float m = fabsf(x);
        int lo = 0, hi = H - 1;
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            if (m >= c.edges[mid]) lo = mid + 1; else hi = mid;
        }
        return (uint32_t)((x > 0.0f) ? H + lo : H - 1 - lo);
    }
};

// One thread encodes 4 consecutive columns (4*BITS bits); 8/BITS neighbouring
// lanes OR their pieces into one 32-bit word and one of them stores it.  Every
// word of the padded row is written (columns >= D encode as 0).
template <class Src, int BITS, typename Coder, bool VEC>
__global__ __launch_bounds__(kThreads) void quantize_sq_kernel(Src src, int64_t rows, int D, int64_t rb,
                                                              Coder coder,
                                                              uint8_t *__restrict__ codes) {
    __shared__ float s_edges[128];
    typename Coder::Ctx ctx;
    constexpr int LG = 8 / BITS;  // lanes per 32-bit word
    const int GW = (int)(2 * rb / BITS);  // 4-column groups per padded row; multiple of 4*LG
    if constexpr (Coder::kEdges) {
        for (int i = threadIdx.x; i < coder.H - 1; i += kThreads) s_edges[i] = coder.T[i];
        __syncthreads();
    }
    const uint32_t total = gridDim.x * kThreads;
    const uint32_t rows_per_pass = total / (uint32_t)GW;
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    if (t >= rows_per_pass * (uint32_t)GW) return;
    const int g = (int)(t % (uint32_t)GW);
    const int col0 = 4 * g;
    coder.prepare(ctx, col0, D);
    if constexpr (Coder::kEdges) ctx.edges = s_edges;
    typename Src::Ctx sctx;
    src.prepare(sctx, col0, D);
    const int sub = g % LG;
    uint32_t *dst_word = reinterpret_cast<uint32_t *>(codes) + (g / LG);
    const int64_t rw = rb / 4;
    // rows interleaved across the grid: a wave's stores stay contiguous (consecutive rows
    // per thread, as in the fit kernel, measured 15 % slower here)
    for (int64_t r = t / GW; r < rows; r += rows_per_pass) {
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (VEC) {
            if (col0 < D) {
                float4 q = src.load4(sctx, r, col0);
                v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 4; k++)
                if (col0 + k < D) v[k] = src.load1(sctx, r, col0 + k);
        }
        uint32_t piece = 0;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            uint32_t q = (col0 + k < D) ? coder.code(ctx, v[k], k) : 0u;
            piece |= q << (BITS * k);
        }
        piece <<= (4 * BITS) * sub;
#pragma unroll
        for (int o = 1; o < LG; o <<= 1) piece |= (uint32_t)__shfl_xor((int)piece, o);
        if (sub == 0) dst_word[r * rw] = piece;
    }
}

template <class Src, typename Coder>
inline void launch_sq(const Src &src, int64_t rows, int D, int64_t rb, int bits, Coder coder,
                      uint8_t *codes, bool vec, hipStream_t s) {
    const int GW = (int)(2 * rb / bits);
    int64_t want = (rows * GW + 3) / 4;
    if (want < GW) want = GW;
    int blocks = blocks_for(want);
    if ((int64_t)blocks * kThreads < GW) blocks = (GW + kThreads - 1) / kThreads;
#define BF_Q(B)                                                                                 \
    if (vec) quantize_sq_kernel<Src, B, Coder, true><<<blocks, kThreads, 0, s>>>(src, rows, D, rb, coder, codes); \
    else quantize_sq_kernel<Src, B, Coder, false><<<blocks, kThreads, 0, s>>>(src, rows, D, rb, coder, codes)
    switch (bits) {
        case 1: BF_Q(1); break;
        case 2: BF_Q(2); break;
        case 4: BF_Q(4); break;
        default: BF_Q(8); break;
    }
#undef BF_Q
}

// ---- launchers over a row source (scalar kinds)
// the per-column range fit (uniform codes); vec: groups of 4 columns per thread
template <class Src>
inline hipError_t launch_fit_minmax_src(bifeat_params *p, const Src &src, int64_t rows, bool vec,
                                        hipStream_t s) {
    const int D = (int)p->D;
    const int VEC = vec ? 4 : 1;
    const int G = (D + VEC - 1) / VEC;
    int64_t want = (rows * G + 7) / 8;  // about 8 rows per thread
    if (want < G) want = G;
    int blocks = blocks_for(want);
    if ((int64_t)blocks * kThreads < G) blocks = (G + kThreads - 1) / kThreads;
    const int use_lds = D <= 8192;
    const size_t shm = use_lds ? sizeof(int32_t) * 2 * (size_t)D : 0;
    if (vec) fit_minmax_kernel<Src, 4><<<blocks, kThreads, shm, s>>>(src, rows, D, G, p->d_fit, use_lds);
    else fit_minmax_kernel<Src, 1><<<blocks, kThreads, shm, s>>>(src, rows, D, G, p->d_fit, use_lds);
    return hipGetLastError();
}

// the fit of the extreme magnitudes (logarithmic codes without clipping)
template <class Src>
inline hipError_t launch_fit_log_src(bifeat_params *p, const Src &src, int64_t rows, bool vec,
                                     hipStream_t s) {
    const int D = (int)p->D;
    const int VEC = vec ? 4 : 1;
    const int G = (D + VEC - 1) / VEC;
    int64_t want = (rows * G + 7) / 8;
    if (want < G) want = G;
    int blocks = blocks_for(want);
    if ((int64_t)blocks * kThreads < G) blocks = (G + kThreads - 1) / kThreads;
    if (vec) fit_log_rows_kernel<Src, 4><<<blocks, kThreads, 0, s>>>(src, rows, D, G, p->d_fit);
    else fit_log_rows_kernel<Src, 1><<<blocks, kThreads, 0, s>>>(src, rows, D, G, p->d_fit);
    return hipGetLastError();
}

// encode + pack `rows` rows of a row source into the packed rows starting at codes_row0
template <class Src>
inline hipError_t launch_quantize_sq_src(bifeat_params *p, const Src &src, int64_t rows,
                                         uint8_t *codes_row0, bool vec, hipStream_t s) {
    const int D = (int)p->D;
    if (p->scheme.kind == BIFEAT_SQ_UNIFORM) {
        UniformCoder c{p->d_min, p->d_inv, (float)((1u << p->scheme.bits) - 1u)};
        launch_sq(src, rows, D, p->rb, p->scheme.bits, c, codes_row0, vec, s);
    } else {
        LogCoder c{p->d_T, 1 << (p->scheme.bits - 1)};
        launch_sq(src, rows, D, p->rb, p->scheme.bits, c, codes_row0, vec, s);
    }
    return hipGetLastError();
}

}  // namespace bf
