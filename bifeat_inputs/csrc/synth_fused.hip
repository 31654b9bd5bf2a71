// The synthetic table as a row source of the library's produced-table interface
// (include/bifeat_produce.hpp): fit and encode straight from the generator, the raw chunk
// never written to memory.  Input data only: the values are those of synth.hip, bit for bit;
// every kernel and all quantizer arithmetic come from the library's header.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "bifeat_produce.hpp"
#include "synth_value.hpp"

namespace {

// rows [row0, row0 + rows) of the table; F16: values rounded to fp16 (the table's storage type)
template <bool F16>
struct SynthSrc {
    uint64_t key;
    float c_z;
    const float *mu, *sigma;
    int64_t row0;
    int D;
    struct Ctx {
        float m[4], s[4];
        int col0;
    };
    __device__ void prepare(Ctx &c, int col0, int Dc) const {
        c.col0 = col0;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            c.m[k] = col0 + k < Dc ? mu[col0 + k] : 0.f;
            c.s[k] = col0 + k < Dc ? sigma[col0 + k] : 0.f;
        }
    }
    __device__ float one(const Ctx &c, uint64_t e, int k) const {
        const float v = bifeat_synth::value(key, e, c_z, c.m[k], c.s[k]);
        return F16 ? __half2float(__float2half_rn(v)) : v;
    }
    __device__ float4 load4(const Ctx &c, int64_t r, int col0) const {
        const uint64_t e0 = (uint64_t)(row0 + r) * (uint64_t)D + (uint64_t)col0;
        return make_float4(one(c, e0, 0), one(c, e0 + 1, 1), one(c, e0 + 2, 2), one(c, e0 + 3, 3));
    }
    __device__ float load1(const Ctx &c, int64_t r, int col) const {
        return one(c, (uint64_t)(row0 + r) * (uint64_t)D + (uint64_t)col, col - c.col0);
    }
};

}  // namespace

// params: the quantizer handle (bifeat_params *); the other arguments as bifeat_synth_fill.
// Return a bifeat_status.
extern "C" int bifeat_synth_fit(void *params, int dtype, int64_t row0, int64_t rows, int D,
                                uint64_t key, float c_z, const float *mu, const float *sigma,
                                void *stream) {
    bifeat_params *p = (bifeat_params *)params;
    if (dtype == 0) return bifeat::fit_update_produced(p, SynthSrc<false>{key, c_z, mu, sigma, row0, D}, rows, stream);
    return bifeat::fit_update_produced(p, SynthSrc<true>{key, c_z, mu, sigma, row0, D}, rows, stream);
}

extern "C" int bifeat_synth_quantize(void *params, int dtype, int64_t row0, int64_t rows, int D,
                                     uint64_t key, float c_z, const float *mu, const float *sigma,
                                     uint8_t *codes, void *stream) {
    bifeat_params *p = (bifeat_params *)params;
    if (dtype == 0)
        return bifeat::quantize_produced(p, SynthSrc<false>{key, c_z, mu, sigma, row0, D}, rows, codes, row0, stream);
    return bifeat::quantize_produced(p, SynthSrc<true>{key, c_z, mu, sigma, row0, D}, rows, codes, row0, stream);
}
