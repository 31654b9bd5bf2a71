// Fused gather + neighbourhood mean for uniform scalar codes (paper Sec. 3.3
// load fused with the aggregation of Appendix A.1).
//
// Uniform codes decode affinely, x' = min_j + q*scale_j, so
//     mean_j = min_j + scale_j * (sum of the neighbours' codes) / n
// exactly: the inner loop only adds integer codes, and it adds them on whole
// 32-bit words of packed codes (SWAR).  A word is split by shift+mask into
// registers whose fields are wide enough to sum several rows without a carry
// into the neighbouring field:
//   level 0 (lane-local): fields of kF0 bits, kN0 registers per word, kCap0 rows;
//   level 1 (combine/stage): fields of kF1 = 2*kF0 bits, kN1 = 2*kN0 registers,
//            kCap1 rows.  Level 0 is folded into level 1 every kCap0 rows.
// In both levels register r, field f of a word holds code number r + f*N.
// The affine map runs once per output element.
//
// Work mapping (wave-centric, no workgroup barriers in the loop): a wavefront
// takes a tile of 64/G consecutive destinations; a destination is owned by
// G = LPR*S lanes: LPR lanes cover one packed row with one 4..16-byte load each
// and S "slots" take every S-th neighbour (S = 1 for the short lists of sampled
// blocks: no cross-lane traffic at all).  Field sums pass through LDS so that
// the tile's output rows - contiguous in memory - are written by the whole
// wave with consecutive 16-byte stores.  A destination whose list is longer
// than `long_thr` is deferred and then processed by the whole wave (S = 64/LPR)
// in rounds of kCap1 rows, integer partial sums parked in its output row.
#include <type_traits>

#include "common.hpp"

namespace bf {

template <int BITS> struct Swar;
template <> struct Swar<8> {
    static constexpr int kF0 = 16, kN0 = 2, kF1 = 16, kN1 = 2;
    static constexpr uint32_t kMask0 = 0x00FF00FFu, kMask1 = 0;
    static constexpr int kCap0 = 257, kCap1 = 257;
};
template <> struct Swar<4> {
    static constexpr int kF0 = 8, kN0 = 2, kF1 = 16, kN1 = 4;
    static constexpr uint32_t kMask0 = 0x0F0F0F0Fu, kMask1 = 0x00FF00FFu;
    static constexpr int kCap0 = 17, kCap1 = 4369;
};
template <> struct Swar<2> {
    static constexpr int kF0 = 4, kN0 = 2, kF1 = 8, kN1 = 4;
    static constexpr uint32_t kMask0 = 0x33333333u, kMask1 = 0x0F0F0F0Fu;
    static constexpr int kCap0 = 5, kCap1 = 85;
};
template <> struct Swar<1> {
    static constexpr int kF0 = 4, kN0 = 4, kF1 = 8, kN1 = 8;
    static constexpr uint32_t kMask0 = 0x11111111u, kMask1 = 0x0F0F0F0Fu;
    static constexpr int kCap0 = 15, kCap1 = 255;
};

enum : uint32_t { F_SKIP = 1u, F_MORE = 2u, F_PREV = 4u, F_EMPTY = 8u };

constexpr int kWaves = kThreads / 64;
#ifndef BF_SWAR_WPE
#define BF_SWAR_WPE 4
#endif
#ifndef BF_SWAR_U
#define BF_SWAR_U 4
#endif

template <int BITS, int CW, bool VEC, typename IT>
__global__ __launch_bounds__(kThreads, BF_SWAR_WPE) void gather_mean_swar_kernel(
    const uint8_t *__restrict__ codes, int64_t rb, const int64_t *__restrict__ indptr,
    const IT *__restrict__ indices, int64_t V, int D, const float *__restrict__ mn,
    const float *__restrict__ sc, float *__restrict__ out, int lpr_log2, int s_log2, int chunks,
    int long_thr, int min_len, int agg_sum) {
    using W = Swar<BITS>;
    constexpr bool kTwoLevel = W::kF1 != W::kF0;
    constexpr int R0 = CW * W::kN0, R1 = CW * W::kN1;
    constexpr int CPW = 32 / BITS;  // codes per word
    constexpr int CPL = CW * CPW;   // columns per lane
    constexpr int U = BF_SWAR_U < W::kCap0 ? BF_SWAR_U : W::kCap0;  // neighbour rows in flight per lane
    constexpr uint32_t FMAX1 = (1u << W::kF1) - 1u;
    static_assert(W::kCap0 >= U, "a lane must be able to add U rows between folds");

    extern __shared__ uint32_t smem[];
    const int Dp = (D + 3) & ~3;
    float *s_mn = reinterpret_cast<float *>(smem);
    float *s_sc = s_mn + Dp;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int stage_per_wave = (64 >> s_log2) * R1;
    float2 *meta = reinterpret_cast<float2 *>(smem + 2 * Dp) + wave * 64;
    uint32_t *stage = smem + 2 * Dp + 2 * 64 * kWaves + wave * stage_per_wave;
    for (int i = threadIdx.x; i < Dp; i += kThreads) {
        s_mn[i] = i < D ? mn[i] : 0.f;
        s_sc[i] = i < D ? sc[i] : 0.f;
    }
    __syncthreads();

    const int LPR = 1 << lpr_log2;
    // filter mode (min_len >= 0: the short-list kernel has taken every list of at
    // most min_len rows): the main pass only scans 64 list lengths per wave and
    // hands each longer list to the whole wave
    const bool scan = min_len >= 0;
    const int g0_log2 = scan ? 0 : lpr_log2 + s_log2;  // lanes per destination in the main pass
    const int dpw_log2 = 6 - g0_log2;       // destinations per wave tile
    const int dpw = 1 << dpw_log2;
    const int64_t tiles = (V + dpw - 1) >> dpw_log2;
    const int nf4 = (D + 3) / 4;
    // walking the tile's float4 granules 64 at a time: (row, granule) advance
    const int step_d = 64 / nf4, step_f = 64 % nf4;
    const int lane_d = lane / nf4, lane_f = lane % nf4;
    const int lane_chunk = lane & (LPR - 1);
    const int64_t n_waves = (int64_t)gridDim.x * kWaves;
    const bool multi_seg = chunks > LPR;  // packed row longer than one pass of LPR lanes

    for (int64_t tile = (int64_t)blockIdx.x * kWaves + wave; tile < tiles; tile += n_waves) {
        const int64_t v_tile = tile << dpw_log2;
        uint64_t hubs = 0;
        for (int mode = 0;; mode = 1) {
            int sl2, ndst;
            int64_t vbase;
            if (mode == 0) {
                sl2 = s_log2;
                vbase = v_tile;
                ndst = (int)min((int64_t)dpw, V - v_tile);
            } else {
                if (!hubs) break;
                const int hl = __ffsll((unsigned long long)hubs) - 1;
                hubs &= hubs - 1;
                sl2 = 6 - lpr_log2;
                vbase = v_tile + (hl >> g0_log2);
                ndst = 1;
            }
            const int g_log2 = (mode == 0 && scan) ? 0 : lpr_log2 + sl2;
            const int S = 1 << sl2, G = 1 << g_log2;
            const int lig = lane & (G - 1);
            const int slot = lig >> lpr_log2;
            const int d_local = lane >> g_log2;
            const bool valid = d_local < ndst;
            int64_t beg = 0, end = 0;
            if (valid) {
                beg = indptr[vbase + d_local];
                end = indptr[vbase + d_local + 1];
            }
            const int64_t n = end - beg;
            const bool is_short = n <= min_len;  // the short-list kernel's destination
            const bool is_long = mode == 0 && (scan ? !is_short : n > long_thr);
            if (mode == 0) hubs = __ballot(valid && is_long && lig == 0);
            if (mode == 0 && scan) continue;  // nothing is accumulated in the scan pass
            // mean: 1/n, applied to the code sum; sum aggregator: n, applied to the column minimum
            const float inv_n = agg_sum ? (float)n : (n > 0 ? 1.0f / (float)n : 0.0f);
            if (is_long || is_short) end = beg;  // whole wave afterwards / other kernel

            for (int cbase = 0; cbase < chunks; cbase += LPR) {
                const int chunk = cbase + lane_chunk;
                const bool chunk_ok = chunk < chunks;
                // lanes past the row's end read chunk 0 (and discard it): always in bounds
                const uint8_t *cptr = codes + (int64_t)(chunk_ok ? chunk : 0) * (CW * 4);
                int round = 0;
                bool more;
                do {
                    const int64_t rbeg = beg + (int64_t)round * W::kCap1;
                    const int64_t rend = min(end, rbeg + (int64_t)W::kCap1);
                    uint32_t l1[R1];
                    // kFold = false: no lane adds more than kCap0 rows, level 1 is only
                    // formed after the loop (and its registers are free during it)
                    auto accumulate = [&](auto fold_tag) {
                        constexpr bool kFold = decltype(fold_tag)::value;
                        uint32_t l0[R0];
#pragma unroll
                        for (int r = 0; r < R0; r++) l0[r] = 0u;
                        if constexpr (kFold) {
#pragma unroll
                            for (int r = 0; r < R1; r++) l1[r] = 0u;
                        }
                        int cnt = 0;
                        for (int64_t e = rbeg + slot; e < rend; e += (int64_t)U * S) {
                            // branch-free: out-of-range slots re-read the list's last row
                            // and are masked, so all U index loads, then all U row loads,
                            // are in flight together
                            uint32_t w[U][CW];
                            IT row[U];
#pragma unroll
                            for (int u = 0; u < U; u++)
                                row[u] = indices[min(e + (int64_t)u * S, rend - 1)];
#pragma unroll
                            for (int u = 0; u < U; u++) load_words<CW>(cptr + (int64_t)row[u] * rb, w[u]);
#pragma unroll
                            for (int u = 0; u < U; u++) {
                                const uint32_t keep = (chunk_ok && e + (int64_t)u * S < rend) ? ~0u : 0u;
#pragma unroll
                                for (int k = 0; k < CW; k++) w[u][k] &= keep;
                            }
                            if constexpr (kFold) {
                                if (cnt + U > W::kCap0) {  // fold level 0 into level 1
#pragma unroll
                                    for (int k = 0; k < CW; k++)
#pragma unroll
                                        for (int i = 0; i < W::kN0; i++) {
                                            const uint32_t a = l0[k * W::kN0 + i];
                                            l1[k * W::kN1 + i] += a & W::kMask1;
                                            l1[k * W::kN1 + W::kN0 + i] += (a >> W::kF0) & W::kMask1;
                                            l0[k * W::kN0 + i] = 0u;
                                        }
                                    cnt = 0;
                                }
                                cnt += U;
                            }
#pragma unroll
                            for (int u = 0; u < U; u++)
#pragma unroll
                                for (int k = 0; k < CW; k++)
#pragma unroll
                                    for (int i = 0; i < W::kN0; i++)
                                        l0[k * W::kN0 + i] += (w[u][k] >> (BITS * i)) & W::kMask0;
                        }
                        if constexpr (kTwoLevel) {
#pragma unroll
                            for (int k = 0; k < CW; k++)
#pragma unroll
                                for (int i = 0; i < W::kN0; i++) {
                                    const uint32_t a = l0[k * W::kN0 + i];
                                    const uint32_t lo = a & W::kMask1, hi = (a >> W::kF0) & W::kMask1;
                                    if constexpr (kFold) {
                                        l1[k * W::kN1 + i] += lo;
                                        l1[k * W::kN1 + W::kN0 + i] += hi;
                                    } else {
                                        l1[k * W::kN1 + i] = lo;
                                        l1[k * W::kN1 + W::kN0 + i] = hi;
                                    }
                                }
                        } else {
#pragma unroll
                            for (int r = 0; r < R1; r++) l1[r] = l0[r];
                        }
                    };
                    if (!kTwoLevel || __all(rend - rbeg <= (int64_t)W::kCap0 * S))
                        accumulate(std::false_type{});
                    else
                        accumulate(std::true_type{});
                    for (int st = LPR; st < G; st <<= 1)
#pragma unroll
                        for (int r = 0; r < R1; r++) l1[r] += (uint32_t)__shfl_xor((int)l1[r], st);

                    more = rend < end;
                    if (slot == 0 && chunk_ok) {
                        uint32_t *sp = stage + (d_local * LPR + lane_chunk) * R1;
#pragma unroll
                        for (int r = 0; r < R1; r++) sp[r] = l1[r];
                    }
                    if (lig == 0) {
                        uint32_t fl = 0;
                        if (!valid || is_long || is_short || (round > 0 && rbeg >= end)) fl |= F_SKIP;
                        if (more) fl |= F_MORE;
                        if (round > 0) fl |= F_PREV;
                        if (n == 0) fl |= F_EMPTY;
                        meta[d_local] = make_float2(inv_n, __uint_as_float(fl));
                    }
                    wave_sync();

                    // ---- the tile's output rows [vbase, vbase+ndst) x this column segment
                    const int col_lo = cbase * CPL;
                    if constexpr (VEC) {
                        // one float4 granule (row d, granule f) of the tile's output span.
                        // Loads are unconditional (clamped in range) so that consecutive
                        // granules overlap their LDS latency; only the store is predicated.
                        float4 *span = reinterpret_cast<float4 *>(out + vbase * D);
                        auto granule = [&](int m, int d, int f, auto rounds_tag) {
                            constexpr bool kRounds = decltype(rounds_tag)::value;
                            const bool in = d < ndst;
                            const int dd = in ? d : 0;
                            const int j0 = 4 * f;
                            const bool seg = !multi_seg || (j0 >= col_lo && j0 < col_lo + LPR * CPL);
                            const int jl = seg ? j0 - col_lo : 0;
                            const float2 md = meta[dd];
                            const uint32_t fl = __float_as_uint(md.y);
                            const int lc = jl / CPL, jj = jl % CPL;
                            const int k = jj / CPW, c = jj % CPW;
                            const uint32_t *sp = stage + ((dd * LPR + lc) * CW + k) * W::kN1;
                            uint32_t sum[4];
                            if constexpr (W::kN1 >= 4) {
                                const int i0 = c % W::kN1, fi = c / W::kN1;
                                const uint4 q = *reinterpret_cast<const uint4 *>(sp + i0);
                                sum[0] = (q.x >> (W::kF1 * fi)) & FMAX1;
                                sum[1] = (q.y >> (W::kF1 * fi)) & FMAX1;
                                sum[2] = (q.z >> (W::kF1 * fi)) & FMAX1;
                                sum[3] = (q.w >> (W::kF1 * fi)) & FMAX1;
                            } else {  // 8-bit codes: one word = 2 registers x 2 fields
                                const uint2 q = *reinterpret_cast<const uint2 *>(sp);
                                sum[0] = q.x & 0xFFFFu;
                                sum[1] = q.y & 0xFFFFu;
                                sum[2] = q.x >> 16;
                                sum[3] = q.y >> 16;
                            }
                            const float4 a = *reinterpret_cast<const float4 *>(s_sc + j0);
                            const float4 b = *reinterpret_cast<const float4 *>(s_mn + j0);
                            const bool write = in && seg && !(fl & F_SKIP);
                            float4 *dst = span + (in ? m : 0);  // granule m of the tile's contiguous span
                            if constexpr (kRounds) {
                                if (write && (fl & F_PREV)) {
                                    const float4 pv = *dst;
                                    sum[0] += __float_as_uint(pv.x);
                                    sum[1] += __float_as_uint(pv.y);
                                    sum[2] += __float_as_uint(pv.z);
                                    sum[3] += __float_as_uint(pv.w);
                                }
                            }
                            const bool empty = fl & F_EMPTY;  // empty list: zero row
                            float4 val;
                            const float ms = agg_sum ? 1.0f : md.x, mb = agg_sum ? md.x : 1.0f;
                            val.x = empty ? 0.f : fmaf(a.x, (float)sum[0] * ms, b.x * mb);
                            val.y = empty ? 0.f : fmaf(a.y, (float)sum[1] * ms, b.y * mb);
                            val.z = empty ? 0.f : fmaf(a.z, (float)sum[2] * ms, b.z * mb);
                            val.w = empty ? 0.f : fmaf(a.w, (float)sum[3] * ms, b.w * mb);
                            if constexpr (kRounds) {
                                if (fl & F_MORE)
                                    val = make_float4(__uint_as_float(sum[0]), __uint_as_float(sum[1]),
                                                      __uint_as_float(sum[2]), __uint_as_float(sum[3]));
                            }
                            // final values stream out; parked partial sums are read back
                            if (write) {
                                if (kRounds && (fl & F_MORE)) *dst = val;
                                else store_stream(dst, val);
                            }
                        };
                        const int n_it = (ndst * nf4 + 63) >> 6;
                        int d = lane_d, f = lane_f;
                        if (mode == 0) {  // short lists: never in rounds
#pragma unroll 2
                            for (int it = 0; it < n_it; it++) {
                                granule(lane + 64 * it, d, f, std::false_type{});
                                d += step_d;
                                f += step_f;
                                if (f >= nf4) {
                                    f -= nf4;
                                    d++;
                                }
                            }
                        } else {
                            for (int it = 0; it < n_it; it++) {
                                granule(lane + 64 * it, d, f, std::true_type{});
                                d += step_d;
                                f += step_f;
                                if (f >= nf4) {
                                    f -= nf4;
                                    d++;
                                }
                            }
                        }
                    } else {
                        // rows not 16-byte aligned: each group writes its own row, scalar stores
                        const float2 md = meta[valid ? d_local : 0];
                        const uint32_t fl = valid ? __float_as_uint(md.y) : (uint32_t)F_SKIP;
                        if (!(fl & F_SKIP)) {
                            const int f4_lo = cbase * (CPL / 4);
                            const int f4_hi = min(nf4, (cbase + LPR) * (CPL / 4));
                            for (int f4 = f4_lo + lig; f4 < f4_hi; f4 += G) {
                                const int j0 = 4 * f4, jl = j0 - col_lo;
                                const int lc = jl / CPL, jj = jl % CPL;
                                const int k = jj / CPW, c = jj % CPW;
                                const uint32_t *sp = stage + ((d_local * LPR + lc) * CW + k) * W::kN1;
                                uint32_t sum[4];
                                if constexpr (W::kN1 >= 4) {
                                    const int i0 = c % W::kN1, fi = c / W::kN1;
#pragma unroll
                                    for (int x = 0; x < 4; x++) sum[x] = (sp[i0 + x] >> (W::kF1 * fi)) & FMAX1;
                                } else {
                                    sum[0] = sp[0] & 0xFFFFu;
                                    sum[1] = sp[1] & 0xFFFFu;
                                    sum[2] = sp[0] >> 16;
                                    sum[3] = sp[1] >> 16;
                                }
                                float *dst = out + (vbase + d_local) * D + j0;
#pragma unroll
                                for (int x = 0; x < 4; x++) {
                                    if (j0 + x >= D) continue;
                                    uint32_t sx = sum[x];
                                    if (fl & F_PREV) sx += __float_as_uint(dst[x]);
                                    float val;
                                    if (fl & F_MORE) val = __uint_as_float(sx);
                                    else if (fl & F_EMPTY) val = 0.f;
                                    else if (agg_sum) val = fmaf(s_sc[j0 + x], (float)sx, s_mn[j0 + x] * md.x);
                                    else val = fmaf(s_sc[j0 + x], (float)sx * md.x, s_mn[j0 + x]);
                                    dst[x] = val;
                                }
                            }
                        }
                    }
                    wave_sync();  // stage and meta are rewritten by the next round / tile
                    round++;
                } while (__any(more));
            }
        }
    }
}

template <int BITS>
static void launch_swar(bifeat_params *p, const MeanCall &c, int vec, int min_len) {
    using W = Swar<BITS>;
    const int64_t rb = p->rb, payload = p->payload, V = c.V, E = c.E;  // row stride / bytes fetched
    // words per lane: every row chunk must be whole; prefer the choice that
    // leaves the fewest idle lanes, then the widest load
    int cw = 4;
    double best_eff = -1.0;
    for (int cand = 4; cand >= 1; cand--) {
        if (payload % (4 * cand)) continue;
        int chunks = (int)(payload / (4 * cand));
        int lpr = pow2ceil(chunks > 64 ? 64 : chunks);
        int passes = (chunks + lpr - 1) / lpr;
        double eff = (double)chunks / ((double)lpr * passes);
        if (eff > best_eff + 1e-9) {
            best_eff = eff;
            cw = cand;
        }
    }
    const int chunks = (int)(payload / (4 * cw));
    const int lpr = pow2ceil(chunks > 64 ? 64 : chunks);
    // slots per destination: about one per 16 neighbours of the average list
    int S = p->opt_mean_slots;
    if (min_len >= 0) S = 1;  // scan mode: 64 list lengths per wave, long lists by the whole wave
    if (S <= 0) {
        const int64_t avg = V > 0 ? E / V : 0;
        S = pow2ceil((int)((avg + 15) / 16 > 64 ? 64 : (avg + 15) / 16));
    }
    S = pow2ceil(S);
    while (lpr * S > 64) S >>= 1;
    int long_thr = 32 * S;
    if (long_thr > W::kCap1) long_thr = W::kCap1;
    const int dpw = min_len >= 0 ? 64 : 64 / (lpr * S);
    const int64_t tiles = (V + dpw - 1) / dpw;
    int64_t want = (tiles + kWaves - 1) / kWaves;
    const int64_t cap = p->opt_mean_blocks > 0 ? p->opt_mean_blocks : (1 << 20);
    int blocks = (int)(want < cap ? want : cap);
    if (blocks < 1) blocks = 1;
    const int Dp = ((int)p->D + 3) & ~3;
    const int R1 = cw * W::kN1;
    const size_t shm = sizeof(uint32_t) * ((size_t)2 * Dp + 2 * 64 * kWaves + (size_t)kWaves * (64 / S) * R1);
#define BF_SK(CWV, VECV, IT)                                                                       \
    gather_mean_swar_kernel<BITS, CWV, VECV, IT><<<blocks, kThreads, shm, c.s>>>(                  \
        c.codes, rb, c.indptr, (const IT *)c.indices, V, (int)p->D, p->d_min, p->d_scale, c.out,   \
        ilog2(lpr), ilog2(S), chunks, long_thr, min_len, c.agg_sum)
#define BF_SW(CWV)                                                                                 \
    do {                                                                                           \
        if (vec) {                                                                                 \
            if (c.idx32) BF_SK(CWV, true, int32_t);                                                \
            else BF_SK(CWV, true, int64_t);                                                        \
        } else {                                                                                   \
            if (c.idx32) BF_SK(CWV, false, int32_t);                                               \
            else BF_SK(CWV, false, int64_t);                                                       \
        }                                                                                          \
    } while (0)
    switch (cw) {
        case 4: BF_SW(4); break;
        case 3: BF_SW(3); break;
        case 2: BF_SW(2); break;
        default: BF_SW(1); break;
    }
#undef BF_SW
#undef BF_SK
}

void launch_gather_mean_swar(bifeat_params *p, const MeanCall &c, int vec, int min_len) {
    switch (p->scheme.bits) {
        case 1: launch_swar<1>(p, c, vec, min_len); break;
        case 2: launch_swar<2>(p, c, vec, min_len); break;
        case 4: launch_swar<4>(p, c, vec, min_len); break;
        default: launch_swar<8>(p, c, vec, min_len); break;
    }
}

}  // namespace bf
