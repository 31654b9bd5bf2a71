// Fused gather + decode + neighbourhood mean (paper Sec. 3.3 load fused with the
// first aggregation of Appendix A.1: g_i = 1/|N(i)| sum_{j in N(i)} g_j).
//
// Uniform scalar codes decode affinely, x' = min_j + q*scale_j, so
//     mean_j = min_j + scale_j * (sum of codes) / n
// exactly: the inner loop only adds integer codes.  It does so on whole 32-bit
// words with several code fields each (SWAR): a word of packed codes is split
// by shift+mask into NR registers whose fields are wide enough (8 or 16 bits)
// to hold the sum of CAP rows without carrying into the neighbour field.  The
// affine map runs once per output element.
//
// Work mapping: a destination is owned by a group of G = LPR*S lanes: LPR lanes
// cover one packed row with a 4..16-byte load each, S "slots" take every S-th
// neighbour; slots are combined with cross-lane adds, the field sums go through
// LDS, and the group then writes the output row with consecutive 16-byte
// stores.  Neighbour lists longer than CAP are processed in rounds whose
// integer partial sums are parked in the output row itself.
//
// Logarithmic and vector codes do not decode affinely; they take the
// float-accumulate kernel at the end of this file (lane = 4 output columns).
#include "common.hpp"

namespace bf {

template <int BITS>
struct Swar {
    static constexpr int FW = (BITS >= 4) ? 16 : 8;  // accumulator field width
    static constexpr int NR = FW / BITS;             // registers per 32-bit word of codes
    static constexpr uint32_t FMAX = (1u << FW) - 1u;
    static constexpr uint32_t CMAX = (1u << BITS) - 1u;
    static constexpr int CAP = (int)(FMAX / CMAX);   // rows a field can sum
    static constexpr uint32_t MASK = (FW == 16) ? (CMAX | (CMAX << 16)) : (CMAX * 0x01010101u);
    // register i, field f of a word holds the sum of code number i + f*NR
};

struct __attribute__((aligned(4))) U3 { uint32_t x, y, z; };

template <int CW>
__device__ inline void load_words(const uint8_t *p, uint32_t *w) {
    if constexpr (CW == 4) {
        uint4 q = *reinterpret_cast<const uint4 *>(p);
        w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    } else if constexpr (CW == 3) {
        U3 q = *reinterpret_cast<const U3 *>(p);
        w[0] = q.x; w[1] = q.y; w[2] = q.z;
    } else if constexpr (CW == 2) {
        uint2 q = *reinterpret_cast<const uint2 *>(p);
        w[0] = q.x; w[1] = q.y;
    } else {
        w[0] = *reinterpret_cast<const uint32_t *>(p);
    }
}

template <int BITS, int CW>
__global__ __launch_bounds__(kThreads) void gather_mean_swar_kernel(
    const uint8_t *__restrict__ codes, int64_t rb, const int64_t *__restrict__ indptr,
    const int64_t *__restrict__ indices, int64_t V, int D, const float *__restrict__ mn,
    const float *__restrict__ sc, float *__restrict__ out, int lpr_log2, int s_log2, int chunks,
    int vec) {
    using W = Swar<BITS>;
    constexpr int R = CW * W::NR;   // accumulator registers per lane
    constexpr int CPW = 32 / BITS;  // codes per word
    constexpr int CPL = CW * CPW;   // columns per lane
    constexpr int U = 4;            // neighbour rows in flight per lane

    extern __shared__ uint32_t smem[];
    const int Dp = (D + 3) & ~3;
    float *s_mn = reinterpret_cast<float *>(smem);
    float *s_sc = s_mn + Dp;
    uint32_t *stage = smem + 2 * Dp;
    for (int i = threadIdx.x; i < Dp; i += kThreads) {
        s_mn[i] = i < D ? mn[i] : 0.f;
        s_sc[i] = i < D ? sc[i] : 0.f;
    }

    const int LPR = 1 << lpr_log2, S = 1 << s_log2, G = LPR * S;
    const int lig = threadIdx.x & (G - 1);
    const int lane_chunk = lig & (LPR - 1);
    const int slot = lig >> lpr_log2;
    const int gib = threadIdx.x >> (lpr_log2 + s_log2);
    const int gpb = kThreads >> (lpr_log2 + s_log2);
    uint32_t *my_stage = stage + gib * (LPR * R);
    const int64_t tiles = (V + gpb - 1) / gpb;
    const int nf4 = (D + 3) / 4;

    for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int64_t v = tile * gpb + gib;
        int64_t beg = 0, end = 0;
        if (v < V) {
            beg = indptr[v];
            end = indptr[v + 1];
        }
        const float inv_n = end > beg ? 1.0f / (float)(end - beg) : 0.0f;
        for (int cbase = 0; cbase < chunks; cbase += LPR) {
            const int chunk = cbase + lane_chunk;
            const bool chunk_ok = chunk < chunks;
            const uint8_t *cptr = codes + (int64_t)chunk * (CW * 4);
            int round = 0, more;
            do {
                const int64_t rbeg = beg + (int64_t)round * W::CAP;
                const int64_t rend = min(end, rbeg + (int64_t)W::CAP);
                uint32_t acc[R];
#pragma unroll
                for (int r = 0; r < R; r++) acc[r] = 0u;
                for (int64_t e = rbeg + slot; e < rend; e += (int64_t)U * S) {
                    uint32_t w[U][CW];
#pragma unroll
                    for (int u = 0; u < U; u++) {
                        const int64_t ee = e + (int64_t)u * S;
                        if (chunk_ok && ee < rend) {
                            load_words<CW>(cptr + indices[ee] * rb, w[u]);
                        } else {
#pragma unroll
                            for (int k = 0; k < CW; k++) w[u][k] = 0u;
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; u++)
#pragma unroll
                        for (int k = 0; k < CW; k++)
#pragma unroll
                            for (int i = 0; i < W::NR; i++)
                                acc[k * W::NR + i] += (w[u][k] >> (BITS * i)) & W::MASK;
                }
                for (int st = LPR; st < G; st <<= 1)
#pragma unroll
                    for (int r = 0; r < R; r++) acc[r] += (uint32_t)__shfl_xor((int)acc[r], st);
                if (slot == 0 && chunk_ok) {
#pragma unroll
                    for (int r = 0; r < R; r++) my_stage[lane_chunk * R + r] = acc[r];
                }
                __syncthreads();
                more = rend < end;
                const bool active = v < V && (round == 0 || rbeg < end);
                if (active) {
                    const int f4_lo = cbase * (CPL / 4);
                    const int f4_hi = min(nf4, (cbase + LPR) * (CPL / 4));
                    for (int f4 = f4_lo + lig; f4 < f4_hi; f4 += G) {
                        const int j0 = 4 * f4;
                        const int jl = j0 - cbase * CPL;
                        const int lc = jl / CPL, jj = jl % CPL;
                        const int k = jj / CPW, c = jj % CPW;
                        const uint32_t *sp = my_stage + (lc * CW + k) * W::NR;
                        uint32_t sum[4];
                        if constexpr (W::NR >= 4) {
                            const int i0 = c % W::NR, f = c / W::NR;
                            const uint4 q = *reinterpret_cast<const uint4 *>(sp + i0);
                            sum[0] = (q.x >> (W::FW * f)) & W::FMAX;
                            sum[1] = (q.y >> (W::FW * f)) & W::FMAX;
                            sum[2] = (q.z >> (W::FW * f)) & W::FMAX;
                            sum[3] = (q.w >> (W::FW * f)) & W::FMAX;
                        } else {  // 8-bit codes: 4 codes per word in two 2x16-bit registers
                            const uint2 q = *reinterpret_cast<const uint2 *>(sp);
                            sum[0] = q.x & 0xFFFFu;
                            sum[1] = q.y & 0xFFFFu;
                            sum[2] = q.x >> 16;
                            sum[3] = q.y >> 16;
                        }
                        float *dst = out + v * D + j0;
                        if (round > 0) {  // add the integer partial sums parked by earlier rounds
#pragma unroll
                            for (int x = 0; x < 4; x++)
                                if (j0 + x < D) sum[x] += __float_as_uint(dst[x]);
                        }
                        float val[4];
#pragma unroll
                        for (int x = 0; x < 4; x++) {
                            if (more) val[x] = __uint_as_float(sum[x]);
                            else val[x] = (end > beg) ? fmaf(s_sc[j0 + x], (float)sum[x] * inv_n, s_mn[j0 + x]) : 0.f;
                        }
                        if (vec) {
                            *reinterpret_cast<float4 *>(dst) = make_float4(val[0], val[1], val[2], val[3]);
                        } else {
#pragma unroll
                            for (int x = 0; x < 4; x++)
                                if (j0 + x < D) dst[x] = val[x];
                        }
                    }
                }
                round++;
            } while (__syncthreads_or(more));
        }
    }
}

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

template <int KIND, int BITS>
__global__ __launch_bounds__(kThreads) void gather_mean_float_kernel(
    const uint8_t *__restrict__ codes, int64_t rb, const int64_t *__restrict__ indptr,
    const int64_t *__restrict__ indices, int64_t V, int D, const float *__restrict__ pa,
    const float *__restrict__ pb, int w, int len, float *__restrict__ out, int vec) {
    __shared__ float s_lut[KIND == MK_LOG ? (1 << BITS) : 1];
    if constexpr (KIND == MK_LOG) {
        for (int i = threadIdx.x; i < (1 << BITS); i += kThreads) s_lut[i] = pa[i];
        __syncthreads();
    }
    const int G = (D + 3) / 4;
    const int64_t total = (int64_t)gridDim.x * kThreads;
    const int64_t per_pass = total / G;
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= per_pass * G) return;
    const int g = (int)(t % G), col0 = 4 * g;
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
        // fp32 sums over runs of kRun neighbours, runs combined in fp64: keeps the
        // rounding error of very long lists far below the 1e-5 budget
        constexpr int kRun = 32;
        double total[4] = {0.0, 0.0, 0.0, 0.0};
        for (int64_t c0 = beg; c0 < end; c0 += kRun) {
            const int64_t c1 = min(end, c0 + kRun);
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
            for (int64_t e = c0; e < c1; e++) {
                const uint8_t *row = codes + indices[e] * rb;
                if constexpr (KIND == MK_UNIFORM || KIND == MK_LOG) {
                    const uint32_t bits = mean_code_bits4<BITS>(row, g);
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        const uint32_t q = (bits >> (BITS * k)) & mask;
                        if constexpr (KIND == MK_UNIFORM) acc[k] += fmaf((float)q, sc[k], mn[k]);
                        else acc[k] += s_lut[q];
                    }
                } else if constexpr (KIND == MK_VQ4) {
                    const int q = row[part[0]];
                    const float4 c = *reinterpret_cast<const float4 *>(pa + ((int64_t)part[0] * len + q) * w + dim[0]);
                    acc[0] += c.x; acc[1] += c.y; acc[2] += c.z; acc[3] += c.w;
                } else {
#pragma unroll
                    for (int k = 0; k < 4; k++)
                        if (col0 + k < D) acc[k] += pa[((int64_t)part[k] * len + row[part[k]]) * w + dim[k]];
                }
            }
#pragma unroll
            for (int k = 0; k < 4; k++) total[k] += (double)acc[k];
        }
        const double inv_nd = end > beg ? 1.0 / (double)(end - beg) : 0.0;
        float acc[4];
#pragma unroll
        for (int k = 0; k < 4; k++) acc[k] = (float)(total[k] * inv_nd);
        const float inv_n = 1.0f;
        float *dst = out + v * D + col0;
        if (vec) {
            *reinterpret_cast<float4 *>(dst) = make_float4(acc[0] * inv_n, acc[1] * inv_n, acc[2] * inv_n, acc[3] * inv_n);
        } else {
#pragma unroll
            for (int k = 0; k < 4; k++)
                if (col0 + k < D) dst[k] = acc[k] * inv_n;
        }
    }
}

static inline int pow2ceil(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}
static inline int ilog2(int x) {
    int l = 0;
    while ((1 << l) < x) l++;
    return l;
}

template <int BITS>
static void launch_swar(bifeat_params *p, const uint8_t *codes, const int64_t *indptr,
                        const int64_t *indices, int64_t V, float *out, int vec, hipStream_t s) {
    using W = Swar<BITS>;
    const int64_t rb = p->rb;
    // words per lane: every row chunk must be whole; prefer the choice that
    // leaves the fewest idle lanes, then the widest load
    int best_cw = 4;
    double best_eff = -1.0;
    for (int cw = 4; cw >= 1; cw--) {
        if (rb % (4 * cw)) continue;
        int chunks = (int)(rb / (4 * cw));
        int lpr = pow2ceil(chunks > 64 ? 64 : chunks);
        int passes = (chunks + lpr - 1) / lpr;
        double eff = (double)chunks / ((double)lpr * passes);
        if (eff > best_eff + 1e-9) {
            best_eff = eff;
            best_cw = cw;
        }
    }
    const int cw = best_cw;
    const int chunks = (int)(rb / (4 * cw));
    const int lpr = pow2ceil(chunks > 64 ? 64 : chunks);
    int S = p->opt_mean_slots > 0 ? p->opt_mean_slots : (16 / lpr > 0 ? 16 / lpr : 1);
    S = pow2ceil(S);
    while (lpr * S > 64) S >>= 1;
    const int gpb = kThreads / (lpr * S);
    const int64_t tiles = (V + gpb - 1) / gpb;
    int blocks = (int)(tiles < (int64_t)kMaxBlocks ? tiles : kMaxBlocks);
    if (p->opt_mean_blocks > 0 && blocks > p->opt_mean_blocks) blocks = p->opt_mean_blocks;
    const int Dp = ((int)p->D + 3) & ~3;
    const int R = cw * W::NR;
    const size_t shm = sizeof(uint32_t) * ((size_t)2 * Dp + (size_t)gpb * lpr * R);
#define BF_SW(CWV)                                                                               \
    gather_mean_swar_kernel<BITS, CWV><<<blocks, kThreads, shm, s>>>(                            \
        codes, rb, indptr, indices, V, (int)p->D, p->d_min, p->d_scale, out, ilog2(lpr), ilog2(S), \
        chunks, vec)
    switch (cw) {
        case 4: BF_SW(4); break;
        case 3: BF_SW(3); break;
        case 2: BF_SW(2); break;
        default: BF_SW(1); break;
    }
#undef BF_SW
}

template <int KIND>
static void launch_float(bifeat_params *p, const uint8_t *codes, const int64_t *indptr,
                         const int64_t *indices, int64_t V, const float *pa, const float *pb,
                         float *out, int vec, hipStream_t s) {
    const int D = (int)p->D, G = (D + 3) / 4;
    int blocks = blocks_for(V * G);
    if ((int64_t)blocks * kThreads < G) blocks = (G + kThreads - 1) / kThreads;
    const int w = p->scheme.vq_width, len = p->scheme.vq_length;
#define BF_FL(B) \
    gather_mean_float_kernel<KIND, B><<<blocks, kThreads, 0, s>>>(codes, p->rb, indptr, indices, V, D, pa, pb, w, len, out, vec)
    switch (p->scheme.bits) {
        case 1: BF_FL(1); break;
        case 2: BF_FL(2); break;
        case 4: BF_FL(4); break;
        default: BF_FL(8); break;
    }
#undef BF_FL
}

hipError_t launch_gather_mean(bifeat_params *p, const uint8_t *codes, const int64_t *indptr,
                              const int64_t *indices, int64_t V, float *out, hipStream_t s) {
    const int D = (int)p->D;
    const int vec = (D % 4 == 0) && ((uintptr_t)out % 16 == 0);
    const int kind = p->scheme.kind;
    if (kind == BIFEAT_SQ_UNIFORM && !p->opt_mean_generic && D <= 2048) {
        switch (p->scheme.bits) {
            case 1: launch_swar<1>(p, codes, indptr, indices, V, out, vec, s); break;
            case 2: launch_swar<2>(p, codes, indptr, indices, V, out, vec, s); break;
            case 4: launch_swar<4>(p, codes, indptr, indices, V, out, vec, s); break;
            default: launch_swar<8>(p, codes, indptr, indices, V, out, vec, s); break;
        }
    } else if (kind == BIFEAT_SQ_UNIFORM) {
        launch_float<MK_UNIFORM>(p, codes, indptr, indices, V, p->d_min, p->d_scale, out, vec, s);
    } else if (kind == BIFEAT_SQ_LOG) {
        launch_float<MK_LOG>(p, codes, indptr, indices, V, p->d_V, nullptr, out, vec, s);
    } else if (p->scheme.vq_width % 4 == 0 && vec) {
        launch_float<MK_VQ4>(p, codes, indptr, indices, V, p->d_cb, nullptr, out, vec, s);
    } else {
        launch_float<MK_VQ>(p, codes, indptr, indices, V, p->d_cb, nullptr, out, vec, s);
    }
    return hipGetLastError();
}

}  // namespace bf
