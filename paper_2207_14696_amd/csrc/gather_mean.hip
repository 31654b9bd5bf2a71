// Fused gather + decode + neighbourhood mean (paper Sec. 3.3 load fused with the
// first aggregation of Appendix A.1: g_i = 1/|N(i)| sum_{j in N(i)} g_j):
// dispatch, and the float-accumulate kernel used for logarithmic and vector
// codes (which do not decode affinely).  Uniform codes take the integer kernel
// in gather_mean_swar.hip.
#include "common.hpp"

namespace bf {

// ---------------------------------------------------------------- float path
// lane = 4 output columns of one destination; neighbours are decoded and
// summed in fp32 one after the other.
enum { MK_UNIFORM = 0, MK_LOG = 1, MK_VQ4 = 2, MK_VQ = 3 };

template <int BITS>
__device__ inline uint32_t mean_code_bits4(const uint8_t *row, int g) {
    if constexpr (BITS == 8) return *reinterpret_cast<const uint32_t *>(row + 4 * g);
    else if constexpr (BITS == 4) return *reinterpret_cast<const uint16_t *>(row + 2 * g);
    else if constexpr (BITS == 2) return row[g];
    else return (uint32_t)(row[g >> 1] >> (4 * (g & 1))) & 0xFu;
}

// vector codes: BITS = 8 or 16 is the width of a stored index
template <int BITS>
__device__ inline int mean_vq_index(const uint8_t *row, int part) {
    if constexpr (BITS == 16) return reinterpret_cast<const uint16_t *>(row)[part];
    else return row[part];
}

template <int KIND, int BITS, bool VEC, typename IT>
__global__ __launch_bounds__(kThreads) void gather_mean_float_kernel(
    const uint8_t *__restrict__ codes, int64_t rb, const int64_t *__restrict__ indptr,
    const IT *__restrict__ indices, int64_t V, int D, const float *__restrict__ pa,
    const float *__restrict__ pb, int w, int len, int agg_sum, int min_len,
    float *__restrict__ out) {
    __shared__ float s_lut[KIND == MK_LOG ? (1 << (BITS & 15)) : 1];
    if constexpr (KIND == MK_LOG) {
        for (int i = threadIdx.x; i < (1 << BITS); i += kThreads) s_lut[i] = pa[i];
        __syncthreads();
    }
    const int G = (D + 3) / 4;
    const uint32_t total = gridDim.x * kThreads;
    const uint32_t per_pass = total / (uint32_t)G;
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    if (t >= per_pass * (uint32_t)G) return;
    const int g = (int)(t % (uint32_t)G), col0 = 4 * g;
    float mn[4], sc[4];
    int part[4], dim[4];
#pragma unroll
    for (int k = 0; k < 4; k++) {
        const bool ok = col0 + k < D;
        if constexpr (KIND == MK_UNIFORM) {
            mn[k] = ok ? pa[col0 + k] : 0.f;
            sc[k] = ok ? pb[col0 + k] : 0.f;
        }
        if constexpr (KIND == MK_VQ4 || KIND == MK_VQ) {
            part[k] = (col0 + k) / w;
            dim[k] = (col0 + k) % w;
        }
    }
    constexpr uint32_t mask = (1u << BITS) - 1u;
    for (int64_t v = t / G; v < V; v += per_pass) {
        const int64_t beg = indptr[v], end = indptr[v + 1];
        if (end - beg <= min_len) continue;  // a short-list kernel's destination
        // fp32 sums over runs of kRun neighbours, runs combined in fp64: keeps the
        // rounding error of very long lists far below the 1e-5 budget
        constexpr int kRun = 32;
        double total[4] = {0.0, 0.0, 0.0, 0.0};
        for (int64_t c0 = beg; c0 < end; c0 += kRun) {
            const int64_t c1 = min(end, c0 + kRun);
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
            for (int64_t e = c0; e < c1; e++) {
                const uint8_t *row = codes + (int64_t)indices[e] * rb;
                if constexpr (KIND == MK_UNIFORM || KIND == MK_LOG) {
                    const uint32_t bits = mean_code_bits4<BITS>(row, g);
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        const uint32_t q = (bits >> (BITS * k)) & mask;
                        if constexpr (KIND == MK_UNIFORM) acc[k] += fmaf((float)q, sc[k], mn[k]);
                        else acc[k] += s_lut[q];
                    }
                } else if constexpr (KIND == MK_VQ4) {
                    const int q = mean_vq_index<BITS>(row, part[0]);
                    const float4 c = *reinterpret_cast<const float4 *>(pa + ((int64_t)part[0] * len + q) * w + dim[0]);
                    acc[0] += c.x; acc[1] += c.y; acc[2] += c.z; acc[3] += c.w;
                } else {
#pragma unroll
                    for (int k = 0; k < 4; k++)
                        if (col0 + k < D) acc[k] += pa[((int64_t)part[k] * len + mean_vq_index<BITS>(row, part[k])) * w + dim[k]];
                }
            }
#pragma unroll
            for (int k = 0; k < 4; k++) total[k] += (double)acc[k];
        }
        const double inv_nd = agg_sum ? 1.0 : (end > beg ? 1.0 / (double)(end - beg) : 0.0);
        float acc[4];
#pragma unroll
        for (int k = 0; k < 4; k++) acc[k] = (float)(total[k] * inv_nd);
        float *dst = out + v * D + col0;
        if constexpr (VEC) {
            store_stream(reinterpret_cast<float4 *>(dst), make_float4(acc[0], acc[1], acc[2], acc[3]));
        } else {
#pragma unroll
            for (int k = 0; k < 4; k++)
                if (col0 + k < D) dst[k] = acc[k];
        }
    }
}

template <int KIND>
static void launch_float(bifeat_params *p, const MeanCall &c, const float *pa, const float *pb,
                         int vec, int min_len = -1) {
    const int D = (int)p->D, G = (D + 3) / 4;
    int blocks = blocks_for(c.V * G);
    if ((int64_t)blocks * kThreads < G) blocks = (G + kThreads - 1) / kThreads;
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
#define BF_FK(B, VECV, IT)                                                                        \
    gather_mean_float_kernel<KIND, B, VECV, IT><<<blocks, kThreads, 0, c.s>>>(                    \
        c.codes, p->rb, c.indptr, (const IT *)c.indices, c.V, D, pa, pb, w, len, c.agg_sum,       \
        min_len, c.out)
#define BF_FL(B)                                                                                  \
    do {                                                                                          \
        if (vec) {                                                                                \
            if (c.idx32) BF_FK(B, true, int32_t);                                                 \
            else BF_FK(B, true, int64_t);                                                         \
        } else {                                                                                  \
            if (c.idx32) BF_FK(B, false, int32_t);                                                \
            else BF_FK(B, false, int64_t);                                                        \
        }                                                                                         \
    } while (0)
    if constexpr (KIND == MK_VQ4 || KIND == MK_VQ) {
        if (p->cbytes == 2) BF_FL(16);
        else BF_FL(8);
    } else {
        switch (p->scheme.bits) {
            case 1: BF_FL(1); break;
            case 2: BF_FL(2); break;
            case 4: BF_FL(4); break;
            default: BF_FL(8); break;
        }
    }
#undef BF_FL
#undef BF_FK
}

// ------------------------------------------------ two rounds, general form
// out[v] = mean over the seed list of v of the means over the outer lists of decoded rows, for
// every kind of code and any list length.  A wave owns a destination; its lanes take 4 output
// columns each (in rounds of 256 columns); an outer list is summed in fp32 runs of kRun rows
// combined in fp64, and the rounds' divisions and the seed list's sum are fp64.
// only_over > 0: the bounded kernel ran first with that bound and left out the destinations
// that have a list longer than it; only those are done here (the wave looks at its seed
// list's entries 64 at a time).
template <int KIND, int BITS, bool VEC>
__global__ __launch_bounds__(kThreads) void gather_mean_2hop_float_kernel(
    const uint8_t *__restrict__ codes, int64_t rb, const int64_t *__restrict__ indptr1,
    const int64_t *__restrict__ indices1, const int64_t *__restrict__ indptr2,
    const int64_t *__restrict__ indices2, int64_t V2, int D, const float *__restrict__ pa,
    const float *__restrict__ pb, int w, int len, int only_over, float *__restrict__ out) {
    __shared__ float s_lut[KIND == MK_LOG ? (1 << (BITS & 15)) : 1];
    if constexpr (KIND == MK_LOG) {
        for (int i = threadIdx.x; i < (1 << BITS); i += kThreads) s_lut[i] = pa[i];
        __syncthreads();
    }
    const int G = (D + 3) / 4;
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
    constexpr uint32_t mask = (1u << BITS) - 1u;
    constexpr int kRun = 32;
    for (int64_t v = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6); v < V2; v += n_waves) {
        const int64_t beg2 = indptr2[v], end2 = indptr2[v + 1];
        if (only_over > 0) {
            bool over = end2 - beg2 > only_over;
            for (int64_t j0 = beg2; !over && j0 < end2; j0 += 64) {
                bool mine = false;
                if (j0 + lane < end2) {
                    const int64_t u = indices2[j0 + lane];
                    mine = indptr1[u + 1] - indptr1[u] > only_over;
                }
                over = __ballot(mine) != 0;
            }
            if (!over) continue;
        }
        for (int g = lane; g < G; g += 64) {
            const int col0 = 4 * g;
            float mn[4], sc[4];
            int part[4], dim[4];
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const bool ok = col0 + k < D;
                if constexpr (KIND == MK_UNIFORM) {
                    mn[k] = ok ? pa[col0 + k] : 0.f;
                    sc[k] = ok ? pb[col0 + k] : 0.f;
                }
                if constexpr (KIND == MK_VQ4 || KIND == MK_VQ) {
                    part[k] = (col0 + k) / w;
                    dim[k] = (col0 + k) % w;
                }
            }
            double outer[4] = {0.0, 0.0, 0.0, 0.0};
            for (int64_t e2 = beg2; e2 < end2; e2++) {
                const int64_t u = indices2[e2];
                const int64_t beg = indptr1[u], end = indptr1[u + 1];
                if (end == beg) continue;  // a zero row
                double total1[4] = {0.0, 0.0, 0.0, 0.0};
                for (int64_t c0 = beg; c0 < end; c0 += kRun) {
                    const int64_t c1 = min(end, c0 + kRun);
                    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
                    for (int64_t e = c0; e < c1; e++) {
                        const uint8_t *row = codes + indices1[e] * rb;
                        if constexpr (KIND == MK_UNIFORM || KIND == MK_LOG) {
                            const uint32_t bits = mean_code_bits4<BITS>(row, g);
#pragma unroll
                            for (int k = 0; k < 4; k++) {
                                const uint32_t q = (bits >> (BITS * k)) & mask;
                                if constexpr (KIND == MK_UNIFORM) acc[k] += fmaf((float)q, sc[k], mn[k]);
                                else acc[k] += s_lut[q];
                            }
                        } else if constexpr (KIND == MK_VQ4) {
                            const int q = mean_vq_index<BITS>(row, part[0]);
                            const float4 c = *reinterpret_cast<const float4 *>(pa + ((int64_t)part[0] * len + q) * w + dim[0]);
                            acc[0] += c.x; acc[1] += c.y; acc[2] += c.z; acc[3] += c.w;
                        } else {
#pragma unroll
                            for (int k = 0; k < 4; k++)
                                if (col0 + k < D) acc[k] += pa[((int64_t)part[k] * len + mean_vq_index<BITS>(row, part[k])) * w + dim[k]];
                        }
                    }
#pragma unroll
                    for (int k = 0; k < 4; k++) total1[k] += (double)acc[k];
                }
                const double inv1 = 1.0 / (double)(end - beg);
#pragma unroll
                for (int k = 0; k < 4; k++) outer[k] += total1[k] * inv1;
            }
            const double inv2 = end2 > beg2 ? 1.0 / (double)(end2 - beg2) : 0.0;
            float res[4];
#pragma unroll
            for (int k = 0; k < 4; k++) res[k] = (float)(outer[k] * inv2);
            float *dst = out + v * D + col0;
            if constexpr (VEC) {
                *reinterpret_cast<float4 *>(dst) = make_float4(res[0], res[1], res[2], res[3]);
            } else {
#pragma unroll
                for (int k = 0; k < 4; k++)
                    if (col0 + k < D) dst[k] = res[k];
            }
        }
    }
}

template <int KIND>
static void launch_2hop_float(bifeat_params *p, const HopCall &c, const float *pa, const float *pb,
                              int vec, int only_over) {
    const int D = (int)p->D;
    const int blocks = blocks_for(c.V2 * 64, 1 << 16);  // a wave per destination
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
#define BF_HF(B)                                                                                   \
    do {                                                                                           \
        if (vec)                                                                                   \
            gather_mean_2hop_float_kernel<KIND, B, true><<<blocks, kThreads, 0, c.s>>>(            \
                c.codes, p->rb, c.indptr1, c.indices1, c.indptr2, c.indices2, c.V2, D, pa, pb, w,  \
                len, only_over, c.out);                                                            \
        else                                                                                       \
            gather_mean_2hop_float_kernel<KIND, B, false><<<blocks, kThreads, 0, c.s>>>(           \
                c.codes, p->rb, c.indptr1, c.indices1, c.indptr2, c.indices2, c.V2, D, pa, pb, w,  \
                len, only_over, c.out);                                                            \
    } while (0)
    if constexpr (KIND == MK_VQ4 || KIND == MK_VQ) {
        if (p->cbytes == 2) BF_HF(16);
        else BF_HF(8);
    } else {
        switch (p->scheme.bits) {
            case 1: BF_HF(1); break;
            case 2: BF_HF(2); break;
            case 4: BF_HF(4); break;
            default: BF_HF(8); break;
        }
    }
#undef BF_HF
}

hipError_t launch_gather_mean_2hop(bifeat_params *p, const HopCall &c) {
    const int D = (int)p->D;
    const int vec = (D % 4 == 0) && ((uintptr_t)c.out % 16 == 0);
    const int kind = p->scheme.kind, bits = p->scheme.bits;
    const bool affine = kind == BIFEAT_SQ_UNIFORM || (kind == BIFEAT_SQ_LOG && bits == 1);
    const bool pair = kind == BIFEAT_SQ_LOG && bits == 2;
    // The register-accumulator form takes lists of at most `thr` entries: the caller's bound
    // (then it runs alone: lists beyond it get NaN rows and raise the status word), or, without
    // one, the longest it can take - the destinations with a longer list are then left to the
    // general kernel, which looks for them.  It keeps row ids and the outer block's list
    // offsets in 32 bits.
    const bool promised = c.max_degree > 0 && c.max_degree <= hop_lean_max_list();
    const int thr = promised ? c.max_degree : hop_lean_max_list();
    int only_over = 0;
    if ((affine || pair) && vec && !p->opt_mean_generic && p->opt_mean_lean && c.max_degree <= hop_lean_max_list() &&
        c.N <= (int64_t)UINT32_MAX && c.E1 <= (int64_t)UINT32_MAX &&
        launch_gather_mean_2hop_lean(p, c, thr, pair, promised)) {
        if (promised) return hipGetLastError();
        only_over = thr;
    }
    if (kind == BIFEAT_SQ_UNIFORM) {
        launch_2hop_float<MK_UNIFORM>(p, c, p->d_min, p->d_scale, vec, only_over);
    } else if (kind == BIFEAT_SQ_LOG) {
        launch_2hop_float<MK_LOG>(p, c, p->d_V, nullptr, vec, only_over);
    } else {
        // codebooks in LDS where the sliced kernels' shapes allow (and the workspace can be had)
        if (vec && p->opt_vq_sliced && launch_gather_mean_2hop_vq_sliced(p, c)) return hipGetLastError();
        const int w = p->scheme.vq_width;
        if (w % 4 == 0 && vec) launch_2hop_float<MK_VQ4>(p, c, p->d_cb, nullptr, vec, only_over);
        else launch_2hop_float<MK_VQ>(p, c, p->d_cb, nullptr, vec, only_over);
    }
    return hipGetLastError();
}

hipError_t launch_gather_mean(bifeat_params *p, const MeanCall &c) {
    const int D = (int)p->D;
    const int64_t V = c.V, E = c.E;
    const int vec = (D % 4 == 0) && ((uintptr_t)c.out % 16 == 0);
    const int kind = p->scheme.kind;
    // With the caller's bound on the list lengths a short-list kernel that covers the bound
    // runs alone: the pass that looks for longer lists is not launched, and a list that breaks
    // the promise gets a row of NaNs and raises the handle's status word.
    const bool promised = c.max_degree > 0;
    // the short-list kernels keep row ids in 32 bits; a table of 2^32 rows or more (possible
    // with 16-byte rows) stays with the general kernels
    const bool ids32 = c.N <= (int64_t)UINT32_MAX;
    const int64_t avg = V > 0 ? E / V : 0;
    const int64_t need = promised ? c.max_degree : 2 * avg;
    // 1-bit logarithmic codes (Sec. 3.1: sign only) decode affinely, V[0] + q*(V[1]-V[0]),
    // so they take the integer-sum kernels of the uniform codes with that map per column
    const bool affine = kind == BIFEAT_SQ_UNIFORM || (kind == BIFEAT_SQ_LOG && p->scheme.bits == 1);
    if (affine && !p->opt_mean_generic && D <= 2048) {
        // Short lists (sampled blocks) go to the lean kernel, anything longer to the
        // general one; each skips the other's destinations.  The caller's bound on
        // the list length (or, without one, twice the average) picks the lean
        // kernel's field width.
        const bool wide = need > lean_capacity(p->scheme.bits, false);
        const int thr = lean_capacity(p->scheme.bits, wide);
        const bool lean = p->opt_mean_lean && p->opt_mean_slots == 0 && vec && V > 0 && need <= thr && ids32 &&
                          launch_gather_mean_lean(p, c, thr, wide, -1, promised);
        const bool all_short = lean && promised;
        if (!all_short) {
            // Without the caller's bound the narrow form was chosen on the average alone: the
            // lists between its capacity and the wide form's (a sampler's fan-out sits there
            // when most lists are full) go to the wide form, not to the general kernel.
            int covered = lean ? thr : -1;
            const int thr_wide = lean_capacity(p->scheme.bits, true);
            if (lean && !wide && thr_wide > thr &&
                launch_gather_mean_lean(p, c, thr_wide, true, thr, false))
                covered = thr_wide;
            launch_gather_mean_swar(p, c, vec, covered);
        }
    } else if (kind == BIFEAT_SQ_UNIFORM) {
        launch_float<MK_UNIFORM>(p, c, p->d_min, p->d_scale, vec);
    } else if (kind == BIFEAT_SQ_LOG && p->scheme.bits == 2 && vec && D <= 1024 && !p->opt_mean_generic) {
        // short lists: the two bit planes summed as integers by the 1-bit short-list kernel;
        // longer lists: the table look-up kernel, each skipping the other's destinations
        const bool wide = need > lean_capacity(1, false);
        const int thr = lean_capacity(1, wide);
        const bool lean = p->opt_mean_lean && V > 0 && need <= thr && ids32 &&
                          launch_gather_mean_lean_log2(p, c, thr, wide, -1, promised);
        const bool all_short = lean && promised;
        if (!all_short) {
            int covered = lean ? thr : -1;
            const int thr_wide = lean_capacity(1, true);
            if (lean && !wide && thr_wide > thr &&
                launch_gather_mean_lean_log2(p, c, thr_wide, true, thr, false))
                covered = thr_wide;
            launch_float<MK_LOG>(p, c, p->d_V, nullptr, vec, covered);
        }
    } else if (kind == BIFEAT_SQ_LOG && (p->scheme.bits == 4 || p->scheme.bits == 8) && vec &&
               !p->opt_mean_generic) {
        // short lists: the look-up kernel with whole 16-byte code loads; longer lists: the
        // general kernel, each skipping the other's destinations
        const int thr = logf_capacity();
        const bool tiled = p->opt_mean_lean && V > 0 && need <= thr && ids32 &&
                           launch_gather_mean_logf(p, c, thr, promised);
        const bool all_short = tiled && promised;
        if (!all_short) launch_float<MK_LOG>(p, c, p->d_V, nullptr, vec, tiled ? thr : -1);
    } else if (kind == BIFEAT_SQ_LOG) {
        launch_float<MK_LOG>(p, c, p->d_V, nullptr, vec);
    } else if (p->opt_vq_sliced && launch_gather_mean_vq_sliced(p, c)) {
        // vector codes, codebook slices in LDS
    } else if (p->scheme.vq_width % 4 == 0 && vec) {
        launch_float<MK_VQ4>(p, c, p->d_cb, nullptr, vec);
    } else {
        launch_float<MK_VQ>(p, c, p->d_cb, nullptr, vec);
    }
    return hipGetLastError();
}

}  // namespace bf
