// Device twin of the host feature generator (bifeat_inputs/features.py): fills
// a [rows x D] chunk of the synthetic table directly in GPU memory, bit for bit
// what the numpy recipe produces.  Input data only: no quantizer arithmetic.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "synth_value.hpp"

namespace {

using bifeat_synth::value;

template <typename T> __device__ inline void store4(T *p, const float v[4]);
template <> __device__ inline void store4<float>(float *p, const float v[4]) {
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ inline void store4<__half>(__half *p, const float v[4]) {
    __half2 a = __halves2half2(__float2half_rn(v[0]), __float2half_rn(v[1]));
    __half2 b = __halves2half2(__float2half_rn(v[2]), __float2half_rn(v[3]));
    uint2 u;
    u.x = *reinterpret_cast<uint32_t *>(&a);
    u.y = *reinterpret_cast<uint32_t *>(&b);
    *reinterpret_cast<uint2 *>(p) = u;
}
template <typename T> __device__ inline T cast1(float v);
template <> __device__ inline float cast1<float>(float v) { return v; }
template <> __device__ inline __half cast1<__half>(float v) { return __float2half_rn(v); }

template <typename T, bool VEC>
__global__ __launch_bounds__(256) void fill_kernel(T *out, int64_t row0, int64_t rows, int D,
                                                  uint64_t key, float c_z, const float *mu,
                                                  const float *sigma) {
    const int G = (D + 3) / 4;
    const int64_t total = (int64_t)gridDim.x * 256;
    const int64_t rows_per_pass = total / G;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= rows_per_pass * G) return;
    const int g = (int)(t % G), col0 = 4 * g;
    float m[4], s[4];
#pragma unroll
    for (int k = 0; k < 4; k++) {
        m[k] = col0 + k < D ? mu[col0 + k] : 0.f;
        s[k] = col0 + k < D ? sigma[col0 + k] : 0.f;
    }
    for (int64_t r = t / G; r < rows; r += rows_per_pass) {
        const uint64_t e0 = (uint64_t)(row0 + r) * (uint64_t)D + (uint64_t)col0;
        float v[4];
#pragma unroll
        for (int k = 0; k < 4; k++) v[k] = value(key, e0 + k, c_z, m[k], s[k]);
        T *dst = out + r * D + col0;
        if (VEC) {
            store4<T>(dst, v);
        } else {
#pragma unroll
            for (int k = 0; k < 4; k++)
                if (col0 + k < D) dst[k] = cast1<T>(v[k]);
        }
    }
}

}  // namespace

// out: device [rows x D] (dtype 0 = fp32, 1 = fp16); mu, sigma: device [D].
// Returns the hipError_t of the launch.
extern "C" int bifeat_synth_fill(void *out, int dtype, int64_t row0, int64_t rows, int D,
                                 uint64_t key, float c_z, const float *mu, const float *sigma,
                                 void *stream) {
    if (rows <= 0) return 0;
    const int G = (D + 3) / 4;
    int64_t want = (rows * G + 255) / 256;
    if (want > 4096) want = 4096;
    if (want * 256 < G) want = (G + 255) / 256;
    const bool vec = D % 4 == 0;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == 0) {
        if (vec) fill_kernel<float, true><<<(int)want, 256, 0, s>>>((float *)out, row0, rows, D, key, c_z, mu, sigma);
        else fill_kernel<float, false><<<(int)want, 256, 0, s>>>((float *)out, row0, rows, D, key, c_z, mu, sigma);
    } else {
        if (vec) fill_kernel<__half, true><<<(int)want, 256, 0, s>>>((__half *)out, row0, rows, D, key, c_z, mu, sigma);
        else fill_kernel<__half, false><<<(int)want, 256, 0, s>>>((__half *)out, row0, rows, D, key, c_z, mu, sigma);
    }
    return (int)hipGetLastError();
}
