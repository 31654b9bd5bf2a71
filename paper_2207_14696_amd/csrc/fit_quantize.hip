// Streaming fit and encode+pack kernels (one-time preprocessing, paper
// Sec. 3.3; code definitions Sec. 3.1 Eq. (1) and Sec. 3.2).
//
// All three kernels stream a row-major [rows x D] chunk once.  A thread owns a
// fixed group of consecutive columns for its whole life (the grid's row stride
// is a multiple of the groups per row), so per-column parameters live in
// registers while consecutive lanes still read consecutive addresses.
#include "common.hpp"

namespace bf {

// ------------------------------------------------------------------ fit state
__global__ void fit_reset_kernel(int32_t *state, int n_half, int32_t a, int32_t b) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_half) {
        state[i] = a;
        state[n_half + i] = b;
    }
}

hipError_t launch_fit_reset(bifeat_params *p, hipStream_t s) {
    if (p->scheme.kind == BIFEAT_SQ_UNIFORM) {
        int D = (int)p->D;
        fit_reset_kernel<<<(D + 255) / 256, 256, 0, s>>>(p->d_fit, D, kKeyPosInf, kKeyNegInf);
    } else {
        // log: [0] = smallest nonzero |x| (bits of +inf), [1] = largest finite |x| (0)
        fit_reset_kernel<<<1, 64, 0, s>>>(p->d_fit, 1, 0x7F800000, 0);
    }
    return hipGetLastError();
}

// per-column min / max of a chunk merged into the running state.
// VEC = 4 needs D % 4 == 0 and a 16-byte (fp16: 8-byte) aligned chunk.
template <typename T, int VEC>
__global__ __launch_bounds__(kThreads) void fit_minmax_kernel(const T *__restrict__ x,
                                                             int64_t rows, int D, int G,
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
        const T *src = x + (int64_t)g * VEC;
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
                float4 q = load4(src + r * D);
                v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
            } else {
                v[0] = load1(src + r * D);
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

// smallest nonzero and largest finite magnitude of a chunk (log scheme);
// positive floats order like their bit patterns
template <typename T, bool VEC>
__global__ __launch_bounds__(kThreads) void fit_log_kernel(const T *__restrict__ x, int64_t n,
                                                          int32_t *state) {
    uint32_t mmin = 0x7F800000u, mmax = 0u;
    auto take = [&](float v) {
        const uint32_t m = __float_as_uint(fabsf(v));
        if (m < 0x7F800000u) {  // finite
            if (m != 0u && m < mmin) mmin = m;
            if (m > mmax) mmax = m;
        }
    };
    if constexpr (VEC) {
        // every workgroup streams one contiguous piece of the chunk, 4 elements per lane
        const int64_t n4 = n >> 2, per_block = (n4 + gridDim.x - 1) / gridDim.x;
        const int64_t i0 = (int64_t)blockIdx.x * per_block, i1 = min(n4, i0 + per_block);
#pragma unroll 4
        for (int64_t i = i0 + threadIdx.x; i < i1; i += kThreads) {
            const float4 v = load4(x + 4 * i);
            take(v.x);
            take(v.y);
            take(v.z);
            take(v.w);
        }
        if (blockIdx.x == 0 && threadIdx.x < (n & 3)) take(load1(x + 4 * n4 + threadIdx.x));
    } else {
        const int64_t stride = (int64_t)gridDim.x * kThreads;
#pragma unroll 4
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride)
            take(load1(x + i));
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

hipError_t launch_fit_update(bifeat_params *p, const void *chunk, int dtype, int64_t rows,
                             hipStream_t s) {
    const int D = (int)p->D;
    if (p->scheme.kind == BIFEAT_SQ_LOG) {
        int64_t n = rows * D;
        int blocks = blocks_for((n + 31) / 32);
        const bool vec4 = (uintptr_t)chunk % (dtype == BIFEAT_F32 ? 16 : 8) == 0;
        if (dtype == BIFEAT_F32) {
            if (vec4) fit_log_kernel<float, true><<<blocks, kThreads, 0, s>>>((const float *)chunk, n, p->d_fit);
            else fit_log_kernel<float, false><<<blocks, kThreads, 0, s>>>((const float *)chunk, n, p->d_fit);
        } else {
            if (vec4) fit_log_kernel<__half, true><<<blocks, kThreads, 0, s>>>((const __half *)chunk, n, p->d_fit);
            else fit_log_kernel<__half, false><<<blocks, kThreads, 0, s>>>((const __half *)chunk, n, p->d_fit);
        }
        return hipGetLastError();
    }
    const size_t esz = dtype == BIFEAT_F32 ? 4 : 2;
    const bool vec = (D % 4 == 0) && ((uintptr_t)chunk % (4 * esz) == 0);
    const int VEC = vec ? 4 : 1;
    const int G = (D + VEC - 1) / VEC;
    int64_t want = (rows * G + 7) / 8;  // about 8 rows per thread
    if (want < G) want = G;
    int blocks = blocks_for(want);
    if ((int64_t)blocks * kThreads < G) blocks = (G + kThreads - 1) / kThreads;
    const int use_lds = D <= 8192;
    const size_t shm = use_lds ? sizeof(int32_t) * 2 * (size_t)D : 0;
#define BF_FIT(T, V) \
    fit_minmax_kernel<T, V><<<blocks, kThreads, shm, s>>>((const T *)chunk, rows, D, G, p->d_fit, use_lds)
    if (dtype == BIFEAT_F32) {
        if (vec) BF_FIT(float, 4); else BF_FIT(float, 1);
    } else {
        if (vec) BF_FIT(__half, 4); else BF_FIT(__half, 1);
    }
#undef BF_FIT
    return hipGetLastError();
}

// scale_j = (max_j - min_j)/L and inv_j = L/(max_j - min_j): fp64 subtraction
// and division, one rounding to fp32; 0 for a constant column; zeros as +0.
__global__ void finalize_uniform_kernel(const int32_t *state, int D, int bits, float *mn,
                                        float *mx, float *scale, float *inv) {
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= D) return;
    float lo = key_float(state[j]), hi = key_float(state[D + j]);
    if (lo == 0.0f) lo = 0.0f;
    if (hi == 0.0f) hi = 0.0f;
    double L = (double)((1u << bits) - 1u);
    double range = (double)hi - (double)lo;
    mn[j] = lo;
    mx[j] = hi;
    if (range > 0.0) {
        scale[j] = (float)(range / L);
        inv[j] = (float)(L / range);
    } else {
        scale[j] = 0.0f;
        inv[j] = 0.0f;
    }
}

hipError_t launch_finalize_uniform(bifeat_params *p, hipStream_t s) {
    int D = (int)p->D;
    finalize_uniform_kernel<<<(D + 255) / 256, 256, 0, s>>>(p->d_fit, D, p->scheme.bits, p->d_min,
                                                            p->d_max, p->d_scale, p->d_inv);
    return hipGetLastError();
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
template <typename T, int BITS, typename Coder, bool VEC>
__global__ __launch_bounds__(kThreads) void quantize_sq_kernel(const T *__restrict__ x,
                                                              int64_t rows, int D, int64_t rb,
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
    const int sub = g % LG;
    uint32_t *dst_word = reinterpret_cast<uint32_t *>(codes) + (g / LG);
    const int64_t rw = rb / 4;
    // rows interleaved across the grid: a wave's stores stay contiguous (consecutive rows
    // per thread, as in the fit kernel, measured 15 % slower here)
    for (int64_t r = t / GW; r < rows; r += rows_per_pass) {
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        const T *src = x + r * D + col0;
        if (VEC) {
            if (col0 < D) {
                float4 q = load4(src);
                v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 4; k++)
                if (col0 + k < D) v[k] = load1(src + k);
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

template <typename T, typename Coder>
static void launch_sq(const T *x, int64_t rows, int D, int64_t rb, int bits, Coder coder,
                      uint8_t *codes, bool vec, hipStream_t s) {
    const int GW = (int)(2 * rb / bits);
    int64_t want = (rows * GW + 3) / 4;
    if (want < GW) want = GW;
    int blocks = blocks_for(want);
    if ((int64_t)blocks * kThreads < GW) blocks = (GW + kThreads - 1) / kThreads;
#define BF_Q(B)                                                                                 \
    if (vec) quantize_sq_kernel<T, B, Coder, true><<<blocks, kThreads, 0, s>>>(x, rows, D, rb, coder, codes); \
    else quantize_sq_kernel<T, B, Coder, false><<<blocks, kThreads, 0, s>>>(x, rows, D, rb, coder, codes)
    switch (bits) {
        case 1: BF_Q(1); break;
        case 2: BF_Q(2); break;
        case 4: BF_Q(4); break;
        default: BF_Q(8); break;
    }
#undef BF_Q
}

// Vector codes (Sec. 3.2): workgroup = one part x strips of 256 rows, thread =
// one row whose sub-vector stays in registers; the part's codebook passes
// through LDS in chunks of EC entries (all of it at once when it fits), read
// by all threads at the same address (broadcast).  Euclidean: fp32, dims
// ascending, subtract / multiply / add rounded separately, strict < keeps the
// lowest index on ties.  Cosine: fp32 dot product accumulated the same way,
// times the entry's reciprocal norm, strict > keeps the lowest index.
// W > 0: the width, known at compile time; W == 0: any width up to WMAX.
template <typename T, int W, int WMAX, int METRIC, typename CODE>
__global__ __launch_bounds__(kThreads) void vq_assign_kernel(
    const T *__restrict__ x, int64_t rows, int D, int w_rt, int len, int P, int EC,
    const float *__restrict__ cb, const float *__restrict__ rnorm, uint8_t *__restrict__ codes,
    int64_t rb) {
    extern __shared__ float s_cb[];
    const int w = W > 0 ? W : w_rt;
    float *s_rn = s_cb + EC * w;
    const int p = blockIdx.x;
    const float *part_cb = cb + (int64_t)p * len * w;
    const bool single = len <= EC;
    auto stage = [&](int e0, int ec) {
        for (int i = threadIdx.x; i < ec * w; i += kThreads) s_cb[i] = part_cb[(int64_t)e0 * w + i];
        if constexpr (METRIC == BIFEAT_VQ_COSINE)
            for (int i = threadIdx.x; i < ec; i += kThreads) s_rn[i] = rnorm[(int64_t)p * len + e0 + i];
    };
    if (single) {
        stage(0, len);
        __syncthreads();
    }
    // every thread of the workgroup walks the same strips (the chunk loads synchronise)
    for (int64_t r0 = (int64_t)blockIdx.y * kThreads; r0 < rows; r0 += (int64_t)gridDim.y * kThreads) {
        const int64_t r = r0 + threadIdx.x;
        const bool valid = r < rows;
        float sub[WMAX];
#pragma unroll
        for (int d = 0; d < WMAX; d++)
            sub[d] = (valid && d < w && p * w + d < D) ? load1(x + r * D + (int64_t)p * w + d) : 0.0f;
        int best = 0;
        float bestv = METRIC == BIFEAT_VQ_COSINE ? -INFINITY : INFINITY;
        for (int e0 = 0; e0 < len; e0 += EC) {
            const int ec = min(EC, len - e0);
            if (!single) {
                __syncthreads();
                stage(e0, ec);
                __syncthreads();
            }
            for (int c = 0; c < ec; c++) {
                const float *ent = s_cb + c * w;
                float acc = 0.0f;
#pragma unroll
                for (int d = 0; d < WMAX; d++) {
                    if (W > 0 || d < w) {  // uniform; sub[] stays in registers
                        if constexpr (METRIC == BIFEAT_VQ_COSINE) {
                            acc = __fadd_rn(acc, __fmul_rn(sub[d], ent[d]));
                        } else {
                            const float diff = __fsub_rn(sub[d], ent[d]);
                            acc = __fadd_rn(acc, __fmul_rn(diff, diff));
                        }
                    }
                }
                if constexpr (METRIC == BIFEAT_VQ_COSINE) {
                    acc = __fmul_rn(acc, s_rn[c]);
                    if (acc > bestv) { bestv = acc; best = e0 + c; }
                } else {
                    if (acc < bestv) { bestv = acc; best = e0 + c; }
                }
            }
        }
        if (valid) {
            reinterpret_cast<CODE *>(codes + r * rb)[p] = (CODE)best;
            if (p == 0)
                for (int64_t b = (int64_t)P * sizeof(CODE); b < rb; b++) codes[r * rb + b] = 0;  // row padding
        }
    }
}

template <typename T, int W, int WMAX>
static void launch_vq_w(bifeat_params *p, const T *x, int64_t rows, uint8_t *codes, int64_t rb,
                        hipStream_t s) {
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
    const bool cosine = p->scheme.vq_metric == BIFEAT_VQ_COSINE;
    int EC = 32768 / (4 * w);  // entries per LDS chunk: 32 KB of entries
    if (EC > len) EC = len;
    int64_t tiles = (rows + kThreads - 1) / kThreads;
    dim3 grid((unsigned)p->P, (unsigned)(tiles > 4096 ? 4096 : tiles));
    const size_t shm = sizeof(float) * ((size_t)EC * w + (cosine ? EC : 0));
#define BF_VQ(M, CODE)                                                                   \
    vq_assign_kernel<T, W, WMAX, M, CODE><<<grid, kThreads, shm, s>>>(                  \
        x, rows, (int)p->D, w, len, p->P, EC, p->d_cb, p->d_rnorm, codes, rb)
    if (p->cbytes == 1) {
        if (cosine) BF_VQ(BIFEAT_VQ_COSINE, uint8_t);
        else BF_VQ(BIFEAT_VQ_L2, uint8_t);
    } else {
        if (cosine) BF_VQ(BIFEAT_VQ_COSINE, uint16_t);
        else BF_VQ(BIFEAT_VQ_L2, uint16_t);
    }
#undef BF_VQ
}

template <typename T>
void launch_vq_assign(bifeat_params *p, const T *x, int64_t rows, uint8_t *codes, int64_t rb,
                      hipStream_t s) {
    const int w = p->scheme.vq_width;
    switch (w) {
        case 1: launch_vq_w<T, 1, 1>(p, x, rows, codes, rb, s); break;
        case 2: launch_vq_w<T, 2, 2>(p, x, rows, codes, rb, s); break;
        case 4: launch_vq_w<T, 4, 4>(p, x, rows, codes, rb, s); break;
        case 8: launch_vq_w<T, 8, 8>(p, x, rows, codes, rb, s); break;
        case 16: launch_vq_w<T, 16, 16>(p, x, rows, codes, rb, s); break;
        default:
            if (w <= 32) launch_vq_w<T, 0, 32>(p, x, rows, codes, rb, s);
            else if (w <= 64) launch_vq_w<T, 0, 64>(p, x, rows, codes, rb, s);
            else launch_vq_w<T, 0, 128>(p, x, rows, codes, rb, s);
            break;
    }
}
template void launch_vq_assign<float>(bifeat_params *, const float *, int64_t, uint8_t *, int64_t,
                                      hipStream_t);
template void launch_vq_assign<__half>(bifeat_params *, const __half *, int64_t, uint8_t *, int64_t,
                                       hipStream_t);

hipError_t launch_quantize(bifeat_params *p, const void *chunk, int dtype, int64_t rows,
                           uint8_t *codes, hipStream_t s) {
    const int D = (int)p->D;
    const size_t esz = dtype == BIFEAT_F32 ? 4 : 2;
    const bool vec = (D % 4 == 0) && ((uintptr_t)chunk % (4 * esz) == 0);
    if (p->scheme.kind == BIFEAT_VQ) {
        if (dtype == BIFEAT_F32) launch_vq_assign(p, (const float *)chunk, rows, codes, p->rb, s);
        else launch_vq_assign(p, (const __half *)chunk, rows, codes, p->rb, s);
    } else if (p->scheme.kind == BIFEAT_SQ_UNIFORM) {
        UniformCoder c{p->d_min, p->d_inv, (float)((1u << p->scheme.bits) - 1u)};
        if (dtype == BIFEAT_F32) launch_sq((const float *)chunk, rows, D, p->rb, p->scheme.bits, c, codes, vec, s);
        else launch_sq((const __half *)chunk, rows, D, p->rb, p->scheme.bits, c, codes, vec, s);
    } else {
        LogCoder c{p->d_T, 1 << (p->scheme.bits - 1)};
        if (dtype == BIFEAT_F32) launch_sq((const float *)chunk, rows, D, p->rb, p->scheme.bits, c, codes, vec, s);
        else launch_sq((const __half *)chunk, rows, D, p->rb, p->scheme.bits, c, codes, vec, s);
    }
    return hipGetLastError();
}

}  // namespace bf
