// The value recipe of the synthetic table on the device (the twin of features.py): element
// e = row * D + col of the table is a pure function of (key, e) and the column's location
// and scale.  Input data only: no quantizer arithmetic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bifeat_synth {

__device__ inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ inline float value(uint64_t key, uint64_t e, float c_z, float mu, float sigma) {
    uint64_t h = mix64(key + e);
    int S = (int)(h & 0xFFFF) + (int)((h >> 16) & 0xFFFF) + (int)((h >> 32) & 0xFFFF) + (int)(h >> 48);
    float z = __fmul_rn((float)(S - 131070), c_z);
    return __fadd_rn(__fmul_rn(sigma, z), mu);
}

}  // namespace bifeat_synth
