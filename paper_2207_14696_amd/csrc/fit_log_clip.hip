// Clipped range for the logarithmic codes (paper Sec. 3.1: e_min / e_max bound
// log2|x| once outliers are clipped; Appendix C calls the clipped fraction a
// minor setting and fixes no rule).  Reading: with n finite nonzero magnitudes
// and clip fraction p, the range ends are the order statistics of |x| at ranks
// floor(p (n-1)) and ceil((1-p) (n-1)) - exactly, not estimated.
//
// Positive floats order like their bit patterns, so an order statistic is found
// by radix selection on the 31 magnitude bits in three passes over the data:
// 11 + 11 + 9 bits.  Each pass histograms the next digit of the values that
// share the digits already fixed (two targets: low and high rank); the host
// walks the histogram between passes.  Counters are 32-bit in LDS (four copies
// against same-bin collisions: the values of a feature table crowd into a few
// exponents) and 64-bit in memory.
#include "common.hpp"

namespace bf {

namespace {

constexpr int kCopies = 4;
// 16 waves share one 64 KB set of histograms, two such workgroups per CU: enough
// waves in flight to keep the read stream going
constexpr int kHistThreads = 1024;

template <typename T, bool VEC>
__global__ __launch_bounds__(kHistThreads) void log_hist_kernel(const T *__restrict__ x, int64_t n,
                                                           int pass, uint32_t prefix_lo,
                                                           uint32_t prefix_hi,
                                                           unsigned long long *__restrict__ hist) {
    __shared__ uint32_t s_h[kCopies][2][kLogHistBins];
    for (int i = threadIdx.x; i < kCopies * 2 * kLogHistBins; i += kHistThreads) (&s_h[0][0][0])[i] = 0u;
    __syncthreads();
    uint32_t(*mine)[kLogHistBins] = s_h[threadIdx.x & (kCopies - 1)];
    auto take = [&](float v) {
        const uint32_t key = __float_as_uint(v) & 0x7FFFFFFFu;
        if (key == 0u || key >= 0x7F800000u) return;  // zero, inf, NaN
        if (pass == 0) {
            atomicAdd(&mine[0][key >> 20], 1u);
        } else if (pass == 1) {
            const uint32_t top = key >> 20, digit = (key >> 9) & 0x7FFu;
            if (top == prefix_lo) atomicAdd(&mine[0][digit], 1u);
            if (top == prefix_hi) atomicAdd(&mine[1][digit], 1u);
        } else {
            const uint32_t top = key >> 9, digit = key & 0x1FFu;
            if (top == prefix_lo) atomicAdd(&mine[0][digit], 1u);
            if (top == prefix_hi) atomicAdd(&mine[1][digit], 1u);
        }
    };
    if constexpr (VEC) {
        // every workgroup streams one contiguous piece of the chunk
        const int64_t n4 = n >> 2, per_block = (n4 + gridDim.x - 1) / gridDim.x;
        const int64_t i0 = (int64_t)blockIdx.x * per_block, i1 = min(n4, i0 + per_block);
#pragma unroll 2
        for (int64_t i = i0 + threadIdx.x; i < i1; i += kHistThreads) {
            const float4 v = load4(x + 4 * i);
            take(v.x);
            take(v.y);
            take(v.z);
            take(v.w);
        }
        if (blockIdx.x == 0 && threadIdx.x < (n & 3)) take(load1(x + 4 * n4 + threadIdx.x));
    } else {
        const int64_t stride = (int64_t)gridDim.x * kHistThreads;
        for (int64_t i = (int64_t)blockIdx.x * kHistThreads + threadIdx.x; i < n; i += stride)
            take(load1(x + i));
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * kLogHistBins; i += kHistThreads) {
        uint32_t c = 0;
#pragma unroll
        for (int k = 0; k < kCopies; k++) c += (&s_h[k][0][0])[i];
        if (c) atomicAdd(&hist[i], (unsigned long long)c);
    }
}

__global__ void log_hist_zero_kernel(unsigned long long *hist) {
    for (int i = threadIdx.x; i < 2 * kLogHistBins; i += blockDim.x) hist[i] = 0ull;
}

}  // namespace

void launch_log_hist_reset(bifeat_params *p, hipStream_t s) {
    log_hist_zero_kernel<<<1, kThreads, 0, s>>>(p->d_hist);
}

hipError_t launch_log_hist_update(bifeat_params *p, const void *chunk, int dtype, int64_t rows,
                                  hipStream_t s) {
    const int64_t n = rows * p->D;
    const size_t esz = dtype == BIFEAT_F32 ? 4 : 2;
    const bool vec = (uintptr_t)chunk % (4 * esz) == 0;
    int64_t want = (n / 32 + kHistThreads - 1) / kHistThreads;
    const int blocks = (int)(want < 1 ? 1 : (want > 1024 ? 1024 : want));  // 2 workgroups per CU (LDS), two rounds
#define BF_LH(T, V)                                                                          \
    log_hist_kernel<T, V><<<blocks, kHistThreads, 0, s>>>((const T *)chunk, n, p->fit_pass,     \
                                                      p->clip_prefix[0], p->clip_prefix[1], p->d_hist)
    if (dtype == BIFEAT_F32) {
        if (vec) BF_LH(float, true); else BF_LH(float, false);
    } else {
        if (vec) BF_LH(__half, true); else BF_LH(__half, false);
    }
#undef BF_LH
    return hipGetLastError();
}

}  // namespace bf
