// Codebook training for the vector codes (paper Sec. 3.2: k-means per part;
// Appendix D: on a uniform row sample, and names the GPU as the place to run it).
//
// Lloyd rounds on a sample chunk resident in GPU memory: initial entries = the
// sample's first `length` rows (per part); each round assigns every sample
// sub-vector to its nearest entry (the same fp32 rule as the encoder, so a
// trained codebook encodes exactly as it was fitted), accumulates per-entry
// sums and counts and replaces each non-empty entry by the mean of its members
// (an entry without members keeps its value).  fp32 atomic accumulation makes
// the result depend on the order of additions in the last bits; it is judged on
// distortion, not bit for bit.
// Two forms: Euclidean one-byte codebooks small enough for LDS fuse the search
// with the accumulation (sums first in LDS per workgroup, then global atomics);
// everything else (cosine metric, up to 16384 entries, wide parts) runs the
// encoder's own kernel into a scratch code array and accumulates from that with
// global atomics.
#include "common.hpp"

namespace bf {

namespace {

// cb[p][c][d] = x[c][p*w + d] for c < len (columns past D read as 0)
template <typename T>
__global__ void vq_init_kernel(const T *__restrict__ x, int D, int w, int len, int P,
                               float *__restrict__ cb) {
    const int64_t n = (int64_t)P * len * w;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int d = (int)(i % w), c = (int)((i / w) % len), p = (int)(i / ((int64_t)w * len));
        const int col = p * w + d;
        cb[i] = col < D ? load1(x + (int64_t)c * D + col) : 0.0f;
    }
}

__global__ void vq_zero_kernel(float *__restrict__ a, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        a[i] = 0.0f;
}

// one workgroup = one part x a strip of sample rows
template <typename T, int W>
__global__ __launch_bounds__(kThreads) void vq_lloyd_accumulate_kernel(
    const T *__restrict__ x, int64_t rows, int D, int w_rt, int len, const float *__restrict__ cb,
    float *__restrict__ sums, float *__restrict__ counts, float *__restrict__ distortion) {
    extern __shared__ float sm[];
    const int w = W > 0 ? W : w_rt;
    float *s_cb = sm, *s_sum = sm + len * w, *s_cnt = s_sum + len * w;
    const int p = blockIdx.x;
    for (int i = threadIdx.x; i < len * w; i += kThreads) {
        s_cb[i] = cb[(int64_t)p * len * w + i];
        s_sum[i] = 0.0f;
    }
    for (int i = threadIdx.x; i < len; i += kThreads) s_cnt[i] = 0.0f;
    __syncthreads();
    float dsum = 0.0f;
    for (int64_t r = (int64_t)blockIdx.y * kThreads + threadIdx.x; r < rows;
         r += (int64_t)gridDim.y * kThreads) {
        const T *src = x + r * D + (int64_t)p * w;
        int best = 0;
        float bestd = INFINITY;
        if constexpr (W > 0) {
            float sub[W];
#pragma unroll
            for (int d = 0; d < W; d++) sub[d] = (p * W + d < D) ? load1(src + d) : 0.0f;
            for (int c = 0; c < len; c++) {
                float dist = 0.0f;
#pragma unroll
                for (int d = 0; d < W; d++) {
                    const float diff = __fsub_rn(sub[d], s_cb[c * W + d]);
                    dist = __fadd_rn(dist, __fmul_rn(diff, diff));
                }
                if (dist < bestd) { bestd = dist; best = c; }
            }
#pragma unroll
            for (int d = 0; d < W; d++) atomicAdd(&s_sum[best * W + d], sub[d]);
        } else {
            for (int c = 0; c < len; c++) {
                float dist = 0.0f;
                for (int d = 0; d < w; d++) {
                    const float xv = (p * w + d < D) ? load1(src + d) : 0.0f;
                    const float diff = __fsub_rn(xv, s_cb[c * w + d]);
                    dist = __fadd_rn(dist, __fmul_rn(diff, diff));
                }
                if (dist < bestd) { bestd = dist; best = c; }
            }
            for (int d = 0; d < w; d++)
                atomicAdd(&s_sum[best * w + d], (p * w + d < D) ? load1(src + d) : 0.0f);
        }
        atomicAdd(&s_cnt[best], 1.0f);
        dsum += bestd;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < len * w; i += kThreads)
        if (s_sum[i] != 0.0f) atomicAdd(&sums[(int64_t)p * len * w + i], s_sum[i]);
    for (int i = threadIdx.x; i < len; i += kThreads)
        if (s_cnt[i] != 0.0f) atomicAdd(&counts[(int64_t)p * len + i], s_cnt[i]);
    for (int o = 32; o > 0; o >>= 1) dsum += __shfl_xor(dsum, o);
    if ((threadIdx.x & 63) == 0) atomicAdd(distortion, dsum);
}

__global__ void vq_lloyd_update_kernel(float *__restrict__ cb, const float *__restrict__ sums,
                                       const float *__restrict__ counts, int w, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const float cnt = counts[i / w];
        if (cnt > 0.0f) cb[i] = sums[i] / cnt;
    }
}

template <typename T>
void lloyd_round(bifeat_params *p, const T *x, int64_t rows, float *dist_slot, hipStream_t s) {
    const int w = p->scheme.vq_width, len = p->scheme.vq_length, P = p->P;
    const int64_t n = (int64_t)P * len * w;
    float *sums = p->d_train, *counts = p->d_train + n;
    vq_zero_kernel<<<256, 256, 0, s>>>(p->d_train, n + (int64_t)P * len);
    int64_t strips = (rows + kThreads * 8 - 1) / (kThreads * 8);  // ~8 rows per thread
    if (strips < 1) strips = 1;
    if (strips > 1024) strips = 1024;
    dim3 grid((unsigned)P, (unsigned)strips);
    const size_t shm = sizeof(float) * ((size_t)2 * len * w + len);
#define BF_LL(W) \
    vq_lloyd_accumulate_kernel<T, W><<<grid, kThreads, shm, s>>>(x, rows, (int)p->D, w, len, p->d_cb, sums, counts, dist_slot)
    switch (w) {
        case 1: BF_LL(1); break;
        case 2: BF_LL(2); break;
        case 4: BF_LL(4); break;
        case 8: BF_LL(8); break;
        case 16: BF_LL(16); break;
        default: BF_LL(0); break;
    }
#undef BF_LL
    vq_lloyd_update_kernel<<<256, 256, 0, s>>>(p->d_cb, sums, counts, w, n);
}

// rnorm[i] = fp32(1 / sqrt(sum_d C_id^2)), 0 for an all-zero entry; sum and root in fp64
__global__ void vq_rnorm_kernel(const float *__restrict__ cb, int64_t entries, int w,
                                float *__restrict__ rnorm) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < entries;
         i += (int64_t)gridDim.x * blockDim.x) {
        double ss = 0.0;
        for (int d = 0; d < w; d++) ss += (double)cb[i * w + d] * (double)cb[i * w + d];
        rnorm[i] = ss > 0.0 ? (float)(1.0 / sqrt(ss)) : 0.0f;
    }
}

// sums / counts / squared distance from a dense code array codes[r][p]
template <typename T, typename CODE>
__global__ __launch_bounds__(kThreads) void vq_accumulate_codes_kernel(
    const T *__restrict__ x, int64_t rows, int D, int w, int len, int P,
    const CODE *__restrict__ codes, const float *__restrict__ cb, float *__restrict__ sums,
    float *__restrict__ counts, float *__restrict__ distortion) {
    const int64_t items = rows * P;
    float dsum = 0.0f;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < items;
         i += (int64_t)gridDim.x * kThreads) {
        const int64_t r = i / P;
        const int p = (int)(i - r * P);
        const int64_t e = (int64_t)p * len + codes[i], ent = e * w;
        for (int d = 0; d < w; d++) {
            const int col = p * w + d;
            const float xv = col < D ? load1(x + r * D + col) : 0.0f;
            atomicAdd(&sums[ent + d], xv);
            const float diff = xv - cb[ent + d];
            dsum += diff * diff;
        }
        atomicAdd(&counts[e], 1.0f);
    }
    for (int o = 32; o > 0; o >>= 1) dsum += __shfl_xor(dsum, o);
    if ((threadIdx.x & 63) == 0) atomicAdd(distortion, dsum);
}

template <typename T>
void lloyd_round_generic(bifeat_params *p, const T *x, int64_t rows, float *dist_slot, hipStream_t s) {
    const int w = p->scheme.vq_width, len = p->scheme.vq_length, P = p->P;
    const int64_t n = (int64_t)P * len * w;
    float *sums = p->d_train, *counts = p->d_train + n;
    vq_zero_kernel<<<1024, 256, 0, s>>>(p->d_train, n + (int64_t)P * len);
    if (p->scheme.vq_metric == BIFEAT_VQ_COSINE) launch_vq_rnorm(p, s);
    launch_vq_assign(p, x, rows, p->d_scratch, (int64_t)P * p->cbytes, s);
    const int blocks = blocks_for(rows * P, 8192);
    if (p->cbytes == 1)
        vq_accumulate_codes_kernel<T, uint8_t><<<blocks, kThreads, 0, s>>>(
            x, rows, (int)p->D, w, len, P, (const uint8_t *)p->d_scratch, p->d_cb, sums, counts, dist_slot);
    else
        vq_accumulate_codes_kernel<T, uint16_t><<<blocks, kThreads, 0, s>>>(
            x, rows, (int)p->D, w, len, P, (const uint16_t *)p->d_scratch, p->d_cb, sums, counts, dist_slot);
    vq_lloyd_update_kernel<<<1024, 256, 0, s>>>(p->d_cb, sums, counts, w, n);
}

}  // namespace

// The handle's workspace (transposed codes of a vector-code gather, code array of the generic
// Lloyd rounds).  It only grows, and a buffer that was handed to kernels is never freed before
// the handle is destroyed: work still in flight, and HIP graphs captured from earlier calls,
// keep a valid address.  While `s` is being captured into a graph nothing is allocated: the
// request then fails unless a call (or bifeat_reserve) at least as large ran before.
bool ensure_scratch(bifeat_params *p, size_t bytes, hipStream_t s) {
    if (p->scratch_bytes >= bytes) return true;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    if (cap != hipStreamCaptureStatusNone) return false;
    void *q = nullptr;
    const size_t want = bytes + bytes / 4;
    if (hipMalloc(&q, want) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    if (p->d_scratch) p->retired.push_back(p->d_scratch);
    p->d_scratch = (uint8_t *)q;
    p->scratch_bytes = want;
    return true;
}

void launch_vq_rnorm(bifeat_params *p, hipStream_t s) {
    const int64_t entries = (int64_t)p->P * p->scheme.vq_length;
    vq_rnorm_kernel<<<blocks_for(entries), kThreads, 0, s>>>(p->d_cb, entries, p->scheme.vq_width,
                                                            p->d_rnorm);
}

// rounds Lloyd iterations over the sample chunk; init = true first seeds the
// codebooks from the chunk's first `length` rows.  d_dist[k] receives the summed
// squared distance of round k's assignment step.
hipError_t launch_vq_train(bifeat_params *p, const void *chunk, int dtype, int64_t rows, bool init,
                           int rounds, hipStream_t s) {
    const int w = p->scheme.vq_width, len = p->scheme.vq_length, P = p->P;
    const bool fused = p->scheme.vq_metric == BIFEAT_VQ_L2 && p->cbytes == 1 &&
                       sizeof(float) * ((size_t)2 * len * w + len) <= 65536;
    if (!fused && !ensure_scratch(p, (size_t)rows * P * p->cbytes, s)) return hipErrorOutOfMemory;
    if (init) {
        if (dtype == BIFEAT_F32)
            vq_init_kernel<float><<<256, 256, 0, s>>>((const float *)chunk, (int)p->D, w, len, P, p->d_cb);
        else
            vq_init_kernel<__half><<<256, 256, 0, s>>>((const __half *)chunk, (int)p->D, w, len, P, p->d_cb);
    }
    vq_zero_kernel<<<1, 64, 0, s>>>(p->d_dist, rounds);
    for (int k = 0; k < rounds; k++) {
        if (fused) {
            if (dtype == BIFEAT_F32) lloyd_round(p, (const float *)chunk, rows, p->d_dist + k, s);
            else lloyd_round(p, (const __half *)chunk, rows, p->d_dist + k, s);
        } else {
            if (dtype == BIFEAT_F32) lloyd_round_generic(p, (const float *)chunk, rows, p->d_dist + k, s);
            else lloyd_round_generic(p, (const __half *)chunk, rows, p->d_dist + k, s);
        }
    }
    return hipGetLastError();
}

}  // namespace bf
