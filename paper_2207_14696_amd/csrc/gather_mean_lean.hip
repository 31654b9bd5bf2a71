// Fused gather + neighbourhood mean for uniform scalar codes, short lists
// (paper Sec. 3.3 load fused with the aggregation of Appendix A.1) - the form
// sampled minibatch blocks take: every destination has at most `fanout`
// neighbours.
//
// Same arithmetic as gather_mean_swar.hip (mean_j = min_j + scale_j*sum(q)/n,
// packed code words added as integers in wide-enough fields), cut down to what
// short lists need so that it fits in few registers and many waves stay
// resident:
//   - LPR lanes own a destination (one 4..16-byte chunk of the packed row each)
//     and walk its whole list: no cross-lane traffic, one level of fields
//     (lists longer than the field capacity `thr` are left to the general
//     kernel, which is launched right after with the complementary filter);
//   - slots past the end of a list load a 16-byte zero row instead of being
//     masked, so the U index loads and then the U row loads of an iteration are
//     all in flight together;
//   - field sums go through LDS once and the tile's output rows (contiguous in
//     memory) are written by the whole wave with consecutive 16-byte stores.
#include "common.hpp"

namespace bf {

static int cap64(int cap) { return cap < 64 ? cap : 64; }

// longest list the short-list kernel takes, in its narrow and wide forms
int lean_capacity(int bits, bool wide) {
    switch (bits) {
        case 8: return cap64(LeanSwar<8, false>::kCap);
        case 4: return cap64(wide ? LeanSwar<4, true>::kCap : LeanSwar<4, false>::kCap);
        case 2: return cap64(LeanSwar<2, false>::kCap);
        default: return cap64(wide ? LeanSwar<1, true>::kCap : LeanSwar<1, false>::kCap);
    }
}

namespace {

#ifndef BF_LEAN_THREADS
#define BF_LEAN_THREADS 256
#endif
constexpr int kLeanThreads = BF_LEAN_THREADS;
constexpr int kLeanWaves = kLeanThreads / 64;
constexpr int kIdxStage = 256;  // list entries a wave parks in LDS per tile
constexpr int kStageMinLprLog2 = 3;  // ... when at least 8 lanes share a destination
#ifndef BF_LEAN_U
#define BF_LEAN_U 4
#endif
#ifndef BF_LEAN_WPE
#define BF_LEAN_WPE 6
#endif

// SUM: the sum aggregator (no division by the list length): meta carries n and
// the column minimum is scaled by it instead.
// PAIR (1-bit fields only): the table is read as 2*D one-bit columns and output
// column t is the sum of the affine maps of bit columns 2t and 2t+1 - the
// 2-bit logarithmic codes, whose decoded sum is linear in the two bit-plane
// sums (see launch_gather_mean_lean_log2).  Dp = number of parameter columns
// (D, or 2*D with PAIR).
// IT: the type of a list entry (int64_t or int32_t).  alone: no other kernel takes the lists
// longer than thr (the caller promised there are none): such a list gets a row of NaNs and
// raises the status word.
// STAGE: the tile's list entries are fetched once by the wave and parked in LDS (see below).
template <int BITS, int CW, bool WIDE, bool SUM, bool PAIR, bool STAGE, typename IT>
__global__ __launch_bounds__(kLeanThreads, BF_LEAN_WPE) void gather_mean_lean_kernel(
    const uint8_t *__restrict__ codes, uint32_t rb, const int64_t *__restrict__ indptr,
    const IT *__restrict__ indices, int64_t V, int D, int Dp, const float *__restrict__ mn,
    const float *__restrict__ sc, const uint8_t *__restrict__ zero_row, float *__restrict__ out,
    int lpr_log2, int chunks, int thr, int lo, int alone, int32_t *__restrict__ status) {
    using W = LeanSwar<BITS, WIDE>;
    constexpr int R = CW * W::kN;   // accumulator registers per lane
    constexpr int CPW = 32 / BITS;  // codes per word
    constexpr int CPL = CW * CPW;   // columns per lane
    constexpr int U = BF_LEAN_U;    // neighbour rows in flight per lane
    constexpr uint32_t FMAX = (1u << W::kF) - 1u;

    extern __shared__ uint32_t smem[];
    float *s_sc = reinterpret_cast<float *>(smem);  // [scale Dp | min Dp], Dp % 4 == 0
    float *s_mn = s_sc + Dp;
    const int lane = threadIdx.x & 63;
    // wave-uniform values kept in scalar registers: the tile bookkeeping runs on the scalar unit
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float *meta = reinterpret_cast<float *>(smem + 2 * Dp) + wave * 64;
    uint32_t *stage = smem + 2 * Dp + 64 * kLeanWaves + wave * (64 * R);
    uint32_t *sidx = smem + 2 * Dp + 64 * kLeanWaves + kLeanWaves * (64 * R) + wave * kIdxStage;

    const int LPR = 1 << lpr_log2;
    const int dpw_log2 = 6 - lpr_log2;
    const int dpw = 1 << dpw_log2;
    const int lane_chunk = lane & (LPR - 1);
    const int d_local = lane >> lpr_log2;
    const bool chunk_ok = lane_chunk < chunks;
    const uint32_t coff = (uint32_t)lane_chunk * (CW * 4);
    const int nf4 = D >> 2;
    const int step_d = 64 / nf4, step_f = 64 % nf4;
    const int lane_d = lane / nf4, lane_f = lane % nf4;
    const int64_t tiles = (V + dpw - 1) >> dpw_log2;
    const int64_t n_waves = (int64_t)gridDim.x * kLeanWaves;

    // list bounds of the destination this lane serves in `tile`
    auto bounds = [&](int64_t tile, int64_t &beg, int64_t &end) {
        const int64_t v = (tile << dpw_log2) + d_local;
        beg = end = 0;
        if (tile < tiles && v < V) {
            beg = indptr[v];
            end = indptr[v + 1];
        }
    };
    int64_t tile = (int64_t)blockIdx.x * kLeanWaves + wave;
    int64_t beg, end;
    bounds(tile, beg, end);  // in flight while the parameters are staged
    for (int i = threadIdx.x; i < Dp; i += kLeanThreads) {
        s_sc[i] = sc[i];
        s_mn[i] = mn[i];
    }
    __syncthreads();

    for (; tile < tiles; tile += n_waves) {
        const int64_t v_tile = tile << dpw_log2;
        const int ndst = (int)min((int64_t)dpw, V - v_tile);
        const int64_t n64 = end - beg;
        // longer lists: the general kernel; lists of up to `lo`: an earlier launch of the narrow form
        const bool mine = d_local < ndst && n64 <= thr && n64 > lo;
        const bool over = alone && d_local < ndst && n64 > thr;  // a broken promise
        if (__ballot(mine || over) == 0) {  // nothing for this launch in the tile
            bounds(tile + n_waves, beg, end);
            continue;
        }
        // STAGE (tables whose rows take 8 or more lanes): the tile's lists are one contiguous
        // run of `indices`; when it is short the wave fetches it once, coalesced, and parks the
        // row ids in LDS (they fit 32 bits: the launcher only takes tables of fewer than 2^32
        // rows), instead of every lane of a destination fetching every entry of its list again.
        // With 1-4 lanes per row the direct fetch is as cheap, and measured faster.
        int64_t tbeg = 0;
        bool staged = false;
        if constexpr (STAGE) {
            tbeg = __shfl(beg, 0);
            const int64_t tlen = __shfl(end, (ndst - 1) << lpr_log2) - tbeg;
            staged = tlen <= kIdxStage;
            if (staged)
                for (int i = lane; i < (int)tlen; i += 64) sidx[i] = (uint32_t)indices[tbeg + i];
        }
        const int n = mine ? (int)n64 : 0;
        if (lane_chunk == 0) {
            // > 0: scale of the sum; 0: empty list; < 0: another kernel's destination; NaN: over
            meta[d_local] = mine ? (n > 0 ? (SUM ? (float)n : 1.0f / (float)n) : 0.0f)
                                 : (over ? __builtin_nanf("") : -1.0f);
            if (over) raise_status(status, kStatusListTooLong);
        }
        if constexpr (STAGE) wave_sync();  // the parked row ids are read next

        uint32_t acc[R];
#pragma unroll
        for (int r = 0; r < R; r++) acc[r] = 0u;
        const int cnt = chunk_ok ? n : 0;
        // U rows per step: their ids first, all together and unconditional (the compiler would
        // otherwise sink each read into a branch on its slot's validity and serialise the row
        // loads behind them), then the U row loads, then the field-parallel adds; slots past
        // the list's end read a zero row
#define BF_LEAN_STEP(ROW_OF)                                                                      \
    for (int k = 0; k < cnt; k += U) {                                                            \
        uint32_t row[U];                                                                          \
        uint32_t w[U][CW];                                                                        \
        _Pragma("unroll") for (int u = 0; u < U; u++) row[u] = (uint32_t)ROW_OF[min(k + u, cnt - 1)]; \
        _Pragma("unroll") for (int u = 0; u < U; u++) asm volatile("" : "+v"(row[u]));            \
        _Pragma("unroll") for (int u = 0; u < U; u++) {                                           \
            const uint8_t *src = (k + u < cnt) ? codes + (uint64_t)row[u] * rb + coff : zero_row; \
            load_words<CW>(src, w[u]);                                                            \
        }                                                                                         \
        _Pragma("unroll") for (int u = 0; u < U; u++)                                             \
            _Pragma("unroll") for (int c = 0; c < CW; c++)                                        \
                _Pragma("unroll") for (int i = 0; i < W::kN; i++)                                 \
                    acc[c * W::kN + i] += (w[u][c] >> (BITS * i)) & W::kMask;                     \
    }
        const IT *ip = indices + beg;
        if constexpr (STAGE) {
            if (staged) {
                const uint32_t *lp = sidx + (int)(beg - tbeg);
                BF_LEAN_STEP(lp)
            } else {
                BF_LEAN_STEP(ip)
            }
        } else {
            BF_LEAN_STEP(ip)
        }
#undef BF_LEAN_STEP
        // the next tile's list bounds travel while this tile's rows are written
        bounds(tile + n_waves, beg, end);
        {
            uint32_t *sp = stage + lane * R;
#pragma unroll
            for (int r = 0; r < R; r++) sp[r] = acc[r];
        }
        wave_sync();

        // ---- the tile's output rows, one contiguous span of ndst*nf4 float4 granules
        float4 *span = reinterpret_cast<float4 *>(out + v_tile * D);
        const int ngran = ndst * nf4;
        int d = lane_d, f = lane_f;
#pragma unroll 2
        for (int m = lane; m < ngran; m += 64) {
            const float md = meta[d];
            const bool some = md > 0.0f;  // md == 0: empty list, zero row
            float4 val;
            if constexpr (PAIR) {
                // 8 consecutive bit columns -> 4 output columns
                const int j0 = 8 * f;
                const int lc = j0 / CPL, jj = j0 % CPL;
                const int k = jj / CPW, c = jj % CPW;  // c % 8 == 0
                const uint32_t *sp = stage + (((d << lpr_log2) + lc) * CW + k) * W::kN;
                uint32_t sum[8];
                if constexpr (W::kN == 4) {  // codes c..c+3 in field c/4, c+4..c+7 in the next
                    const uint4 q = *reinterpret_cast<const uint4 *>(sp);
                    const int sh = W::kF * (c / 4);
                    sum[0] = (q.x >> sh) & FMAX; sum[1] = (q.y >> sh) & FMAX;
                    sum[2] = (q.z >> sh) & FMAX; sum[3] = (q.w >> sh) & FMAX;
                    sum[4] = (q.x >> (sh + W::kF)) & FMAX; sum[5] = (q.y >> (sh + W::kF)) & FMAX;
                    sum[6] = (q.z >> (sh + W::kF)) & FMAX; sum[7] = (q.w >> (sh + W::kF)) & FMAX;
                } else {  // kN == 8: codes c..c+7 in registers 0..7, field c/8
                    const uint4 qa = *reinterpret_cast<const uint4 *>(sp);
                    const uint4 qb = *reinterpret_cast<const uint4 *>(sp + 4);
                    const int sh = W::kF * (c / 8);
                    sum[0] = (qa.x >> sh) & FMAX; sum[1] = (qa.y >> sh) & FMAX;
                    sum[2] = (qa.z >> sh) & FMAX; sum[3] = (qa.w >> sh) & FMAX;
                    sum[4] = (qb.x >> sh) & FMAX; sum[5] = (qb.y >> sh) & FMAX;
                    sum[6] = (qb.z >> sh) & FMAX; sum[7] = (qb.w >> sh) & FMAX;
                }
                const float4 a0 = *reinterpret_cast<const float4 *>(s_sc + j0);
                const float4 a1 = *reinterpret_cast<const float4 *>(s_sc + j0 + 4);
                const float4 b0 = *reinterpret_cast<const float4 *>(s_mn + j0);
                const float4 b1 = *reinterpret_cast<const float4 *>(s_mn + j0 + 4);
                const float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
                const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
                float v[8];
#pragma unroll
                for (int i = 0; i < 8; i++)
                    v[i] = SUM ? fmaf(a[i], (float)sum[i], b[i] * md) : fmaf(a[i], (float)sum[i] * md, b[i]);
                val.x = some ? v[0] + v[1] : 0.0f;
                val.y = some ? v[2] + v[3] : 0.0f;
                val.z = some ? v[4] + v[5] : 0.0f;
                val.w = some ? v[6] + v[7] : 0.0f;
            } else {
            const int j0 = 4 * f;
            const int lc = j0 / CPL, jj = j0 % CPL;
            const int k = jj / CPW, c = jj % CPW;
            const uint32_t *sp = stage + (((d << lpr_log2) + lc) * CW + k) * W::kN;
            uint32_t sum[4];
            if constexpr (W::kN >= 4) {
                const uint4 q = *reinterpret_cast<const uint4 *>(sp + c % W::kN);
                const int sh = W::kF * (c / W::kN);
                sum[0] = (q.x >> sh) & FMAX;
                sum[1] = (q.y >> sh) & FMAX;
                sum[2] = (q.z >> sh) & FMAX;
                sum[3] = (q.w >> sh) & FMAX;
            } else {
                const uint2 q = *reinterpret_cast<const uint2 *>(sp);
                const int sh = W::kF * (c / 2);
                sum[0] = (q.x >> sh) & FMAX;
                sum[1] = (q.y >> sh) & FMAX;
                sum[2] = (q.x >> (sh + W::kF)) & FMAX;
                sum[3] = (q.y >> (sh + W::kF)) & FMAX;
            }
            const float4 a = *reinterpret_cast<const float4 *>(s_sc + j0);
            const float4 b = *reinterpret_cast<const float4 *>(s_mn + j0);
            if constexpr (SUM) {
                val.x = some ? fmaf(a.x, (float)sum[0], b.x * md) : 0.0f;
                val.y = some ? fmaf(a.y, (float)sum[1], b.y * md) : 0.0f;
                val.z = some ? fmaf(a.z, (float)sum[2], b.z * md) : 0.0f;
                val.w = some ? fmaf(a.w, (float)sum[3], b.w * md) : 0.0f;
            } else {
                val.x = some ? fmaf(a.x, (float)sum[0] * md, b.x) : 0.0f;
                val.y = some ? fmaf(a.y, (float)sum[1] * md, b.y) : 0.0f;
                val.z = some ? fmaf(a.z, (float)sum[2] * md, b.z) : 0.0f;
                val.w = some ? fmaf(a.w, (float)sum[3] * md, b.w) : 0.0f;
            }
            }
            if (md != md) val.x = val.y = val.z = val.w = md;  // list beyond the promised bound
            if (!(md < 0.0f)) store_stream(&span[m], val);  // md < 0: not this kernel's destination
            d += step_d;
            f += step_f;
            if (f >= nf4) {
                f -= nf4;
                d++;
            }
        }
        wave_sync();  // stage / meta are rewritten by the next tile
    }
}

template <int BITS, bool WIDE, bool PAIR>
bool launch_lean_bits(bifeat_params *p, const MeanCall &c, int thr, int lo, bool alone,
                      const float *mn, const float *sc) {
    using W = LeanSwar<BITS, WIDE>;
    const int64_t V = c.V;
    const int64_t rb = p->rb, payload = p->payload;  // row stride / bytes the lanes fetch
    int cw = 0;
    double best_eff = -1.0;
    for (int cand = 4; cand >= 1; cand--) {
        if (payload % (4 * cand)) continue;
        const int chunks = (int)(payload / (4 * cand));
        if (chunks > 64) continue;
        const double eff = (double)chunks / pow2ceil(chunks);
        if (eff > best_eff + 1e-9) {
            best_eff = eff;
            cw = cand;
        }
    }
    if (!cw) return false;  // packed row longer than 64 lane loads
    const int chunks = (int)(payload / (4 * cw));
    const int lpr = pow2ceil(chunks);
    const int dpw = 64 / lpr;
    const int64_t tiles = (V + dpw - 1) / dpw;
    const int64_t cap = p->opt_mean_blocks > 0 ? p->opt_mean_blocks : (1 << 16);
    int64_t want = (tiles + kLeanWaves - 1) / kLeanWaves;
    const int blocks = (int)(want < cap ? (want < 1 ? 1 : want) : cap);
    const int D = (int)p->D, Dp = PAIR ? 2 * D : D;
    const int R = cw * W::kN;
    const size_t shm = sizeof(uint32_t) * ((size_t)2 * Dp + 64 * kLeanWaves + (size_t)kLeanWaves * 64 * R +
                                           (size_t)kLeanWaves * kIdxStage);
    const bool stage = ilog2(lpr) >= kStageMinLprLog2;
#define BF_LK(CWV, SUMV, STG, IT)                                                                  \
    gather_mean_lean_kernel<BITS, CWV, WIDE, SUMV, PAIR, STG, IT><<<blocks, kLeanThreads, shm, c.s>>>( \
        c.codes, (uint32_t)rb, c.indptr, (const IT *)c.indices, V, D, Dp, mn, sc, p->d_zero,       \
        c.out, ilog2(lpr), chunks, thr, lo, alone ? 1 : 0, c.status)
#define BF_LS(CWV, SUMV)                                                                           \
    do {                                                                                           \
        if (stage) {                                                                               \
            if (c.idx32) BF_LK(CWV, SUMV, true, int32_t);                                          \
            else BF_LK(CWV, SUMV, true, int64_t);                                                  \
        } else {                                                                                   \
            if (c.idx32) BF_LK(CWV, SUMV, false, int32_t);                                         \
            else BF_LK(CWV, SUMV, false, int64_t);                                                 \
        }                                                                                          \
    } while (0)
#define BF_LN(CWV)                                                                                 \
    do {                                                                                           \
        if (c.agg_sum) BF_LS(CWV, true);                                                           \
        else BF_LS(CWV, false);                                                                    \
    } while (0)
    switch (cw) {
        case 4: BF_LN(4); break;
        case 3: BF_LN(3); break;
        case 2: BF_LN(2); break;
        default: BF_LN(1); break;
    }
#undef BF_LN
#undef BF_LS
#undef BF_LK
    return true;
}

}  // namespace

// Launches the short-list kernel (lists of more than `lo` and at most `thr` rows; wide =
// the form with the larger field capacity); returns false (nothing launched) when the
// table's shape is outside what it handles.
bool launch_gather_mean_lean(bifeat_params *p, const MeanCall &c, int thr, bool wide, int lo,
                             bool alone) {
    const float *mn = p->d_min, *sc = p->d_scale;
    switch (p->scheme.bits) {
        case 1:
            return wide ? launch_lean_bits<1, true, false>(p, c, thr, lo, alone, mn, sc)
                        : launch_lean_bits<1, false, false>(p, c, thr, lo, alone, mn, sc);
        case 2: return launch_lean_bits<2, false, false>(p, c, thr, lo, alone, mn, sc);
        case 4:
            return wide ? launch_lean_bits<4, true, false>(p, c, thr, lo, alone, mn, sc)
                        : launch_lean_bits<4, false, false>(p, c, thr, lo, alone, mn, sc);
        default: return launch_lean_bits<8, false, false>(p, c, thr, lo, alone, mn, sc);
    }
}

// 2-bit logarithmic codes (Sec. 3.1 Eq. (1)/(2) with k = 2): code q = 2*b1 + b0 decodes to
// -v1, -v0, +v0, +v1, so the decoded sum over a list of n rows is
//   v0*(S1 - S0) + v1*(S1 + S0 - n),   S0 = sum of b0, S1 = sum of b1,
// i.e. (v1 - v0)*S0 - n*v1  +  (v0 + v1)*S1: linear in the two bit-plane sums.  The packed row
// is therefore read as 2*D one-bit columns (bit 2t = b0, bit 2t+1 = b1 of column t) by the
// 1-bit kernel, with those two affine maps as per-bit-column parameters (p->d_min / d_scale,
// 2*D entries each), and the epilogue adds each pair.
bool launch_gather_mean_lean_log2(bifeat_params *p, const MeanCall &c, int thr, bool wide, int lo,
                                  bool alone) {
    return wide ? launch_lean_bits<1, true, true>(p, c, thr, lo, alone, p->d_min, p->d_scale)
                : launch_lean_bits<1, false, true>(p, c, thr, lo, alone, p->d_min, p->d_scale);
}

}  // namespace bf
