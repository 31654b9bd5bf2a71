// Streaming fit and encode+pack kernels (one-time preprocessing, paper
// Sec. 3.3; code definitions Sec. 3.1 Eq. (1) and Sec. 3.2).
//
// All three kernels stream a row-major [rows x D] chunk once.  A thread owns a
// fixed group of consecutive columns for its whole life (the grid's row stride
// is a multiple of the groups per row), so per-column parameters live in
// registers while consecutive lanes still read consecutive addresses.
#include "common.hpp"
#include "stream_kernels.hpp"

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
    if (dtype == BIFEAT_F32) return launch_fit_minmax_src(p, ChunkSrc<float>{(const float *)chunk, D}, rows, vec, s);
    return launch_fit_minmax_src(p, ChunkSrc<__half>{(const __half *)chunk, D}, rows, vec, s);
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
    } else if (dtype == BIFEAT_F32) {
        return launch_quantize_sq_src(p, ChunkSrc<float>{(const float *)chunk, D}, rows, codes, vec, s);
    } else {
        return launch_quantize_sq_src(p, ChunkSrc<__half>{(const __half *)chunk, D}, rows, codes, vec, s);
    }
    return hipGetLastError();
}

}  // namespace bf
