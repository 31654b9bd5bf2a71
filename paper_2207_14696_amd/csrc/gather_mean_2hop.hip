// Two rounds of neighbourhood averaging straight from the packed table (Appendix A.1:
// g_i = 1/|N(i)| sum_{j in N(i)} g_j applied twice with nothing in between - the linear
// propagation its error analysis is written for): out[v] = mean over the seed block's list
// of v of the means over the outer block's lists of decoded rows.  The first round's fp32
// rows are never written: the kernel fetches, per entry u of a seed list, the packed rows of
// u's own list, sums their codes as integers in packed fields (as the one-round short-list
// kernel does), and adds (field sum)/|N1(u)| into per-column fp32 accumulators that stay in
// registers; the affine decode is applied once per output element:
//   out[v, j] = min_j * (#non-empty N1(u))/|N2(v)| + scale_j * (1/|N2(v)|) sum_u S_u[j]/|N1(u)|.
//
// This form needs the caller's bound on the list lengths (at most 64): every list sum then
// fits one field (4-bit codes: lists of 18 to 32 rows as two pieces in narrow fields) and a
// destination adds at most 64 terms in fp32 (relative error below 66 * 2^-24 of a sum of
// non-negative terms).  Anything else takes the general kernel in gather_mean.hip.
// A wave's time is a chain of dependent fetches (seed list -> outer lists' bounds -> row ids
// -> rows), so the kernel lives on resident waves: what was measured to matter is one wave
// per workgroup, no register spills, and the cheapest field form the bound allows.
#include "common.hpp"

namespace bf {
namespace {

#ifndef BF_HOP_THREADS
#define BF_HOP_THREADS 64
#endif
// one wave per workgroup: the waves' running times differ by an order of magnitude (they follow
// the destinations' list lengths), and a workgroup's wave slots are only reused together
constexpr int kHopThreads = BF_HOP_THREADS;
constexpr int kHopWaves = kHopThreads / 64;
constexpr int kHopIds = 256;  // row ids a wave parks in LDS at a time: 4 per lane
constexpr int kHopPiece = 16;  // rows per piece of a split list
// build-time switches for A/B measurements (the defaults are what was measured best)
#ifndef BF_HOP_SPLIT
#define BF_HOP_SPLIT 1  // heavy destinations first
#endif
#ifndef BF_HOP_SPLIT16
#define BF_HOP_SPLIT16 1  // 4-bit lists of 18..32 rows as two narrow-field pieces
#endif
#ifndef BF_HOP_U
#define BF_HOP_U 4
#endif
#ifndef BF_HOP_WPE
#define BF_HOP_WPE 4
#endif

// Lane layout: LPR lanes share one packed row (CW words each) and form a group; G2 groups share
// a destination v and take every G2-th entry of its seed list; their accumulators are added
// across the groups at the end.  A wave serves 64 / (LPR * G2) destinations.
// PAIR: 2-bit logarithmic codes read as 2*D one-bit columns whose affine maps add pairwise
// (see launch_gather_mean_lean_log2); Dp = number of parameter columns (D, or 2*D).
// SPLIT: outer lists of more than kHopPiece rows are summed as two pieces, each within what a
// narrow field holds (the bound is then at most 2 * kHopPiece, and a destination still adds at
// most 64 fp32 terms); cheaper per row than the wide fields.
template <int BITS, int CW, bool WIDE, bool PAIR, bool SPLIT>
__global__ __launch_bounds__(kHopThreads, (BITS == 4 && CW == 4 && WIDE) ? 3 : BF_HOP_WPE) void gather_mean_2hop_lean_kernel(
    const uint8_t *__restrict__ codes, uint32_t rb, const int64_t *__restrict__ indptr1,
    const int64_t *__restrict__ indices1, const int64_t *__restrict__ indptr2,
    const int64_t *__restrict__ indices2, int64_t V2, int D, int Dp, const float *__restrict__ mn,
    const float *__restrict__ sc, const uint8_t *__restrict__ zero_row, float *__restrict__ out,
    int lpr_log2, int g2_log2, int chunks, int thr, int heavy, int alone, int32_t *__restrict__ status) {
    using W = LeanSwar<BITS, WIDE>;
    constexpr int R = CW * W::kN;    // field registers per lane
    constexpr int CPW = 32 / BITS;   // codes per word
    constexpr int CPL = CW * CPW;    // columns per lane
    constexpr int FPR = 32 / W::kF;  // fields per register
    constexpr int U = BF_HOP_U;      // rows in flight per lane
    constexpr uint32_t FMAX = (1u << W::kF) - 1u;

    extern __shared__ uint32_t smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int LPR = 1 << lpr_log2, G2 = 1 << g2_log2;
    const int vl_log2 = lpr_log2 + g2_log2, VL = 1 << vl_log2;  // lanes per destination
    const int vpw_log2 = 6 - vl_log2, vpw = 1 << vpw_log2;      // destinations per wave
    const int sub = lane & (LPR - 1);                           // this lane's piece of a packed row
    const int q = (lane >> lpr_log2) & (G2 - 1);                // its group among the destination's
    const int vslot = lane >> vl_log2;
    const int lv = lane & (VL - 1);
    const int ROUND = 4 * LPR;  // row ids a group parks at a time
    uint32_t *sidx = smem + wave * kHopIds + (lane >> lpr_log2) * ROUND;
    // per destination, for every piece of work (the outer list of a seed-list entry, or one of
    // its two pieces): x = where its row ids start, y = rows | whole list's length << 8 |
    // (first piece) << 16
    uint2 *smeta = reinterpret_cast<uint2 *>(smem + kHopWaves * kHopIds) +
                   (wave * vpw + vslot) * (SPLIT ? 2 * thr : thr);
    const bool chunk_ok = sub < chunks;
    const uint32_t coff = (uint32_t)sub * (CW * 4);
    const uint64_t vmask = (VL == 64 ? ~0ull : ((1ull << VL) - 1ull)) << (vslot << vl_log2);
    const int64_t tiles = (V2 + vpw - 1) >> vpw_log2;
    const int64_t n_waves = (int64_t)gridDim.x * kHopWaves;

    // Work per destination varies with its list lengths, and a wave's time is a chain of
    // dependent fetches: with `heavy` > 0 every tile is visited twice, the first time (waves
    // that are dispatched first) to be done only if one of its seed lists has more than
    // `heavy` entries, the second time only if none has - long destinations start early and
    // the short ones fill in behind them.
    const int64_t visits = heavy > 0 ? 2 * tiles : tiles;
    for (int64_t visit = (int64_t)blockIdx.x * kHopWaves + wave; visit < visits; visit += n_waves) {
        const bool second = visit >= tiles;
        const int64_t tile = second ? visit - tiles : visit;
        const int64_t v = (tile << vpw_log2) + vslot;
        const bool valid = v < V2;
        int64_t b2 = 0, e2 = 0;
        if (valid) {
            b2 = indptr2[v];
            e2 = indptr2[v + 1];
        }
        if (heavy > 0 && (__ballot(e2 - b2 > heavy) != 0) == second) continue;
        bool bad = e2 - b2 > thr;  // a list beyond the promised bound
        const int n2 = bad ? 0 : (int)(e2 - b2);
        int npiece = n2;
        for (int j0 = 0; __ballot(j0 + lv < n2) != 0; j0 += VL) {
            const int j = j0 + lv;
            uint32_t b1 = 0u, len = 0u;
            if (j < n2) {
                const int64_t u = indices2[b2 + j];
                const int64_t beg = indptr1[u], end = indptr1[u + 1];
                const bool over = end - beg > thr;
                bad |= over;
                b1 = (uint32_t)beg;
                len = over ? 0u : (uint32_t)(end - beg);
                const uint32_t head = SPLIT ? min(len, (uint32_t)kHopPiece) : len;
                smeta[j] = make_uint2(b1, head | (len << 8) | (1u << 16));
            }
            if constexpr (SPLIT) {
                // second pieces go behind the n2 first ones, in the order of their entries
                const bool more = len > (uint32_t)kHopPiece;
                const uint64_t mine = (__ballot(more) & vmask) >> (vslot << vl_log2);
                if (more)
                    smeta[npiece + __popcll(mine & ((1ull << lv) - 1ull))] =
                        make_uint2(b1 + kHopPiece, (len - kHopPiece) | (len << 8));
                npiece += __popcll(mine);
            }
        }
        wave_sync();

        float facc[CPL];
#pragma unroll
        for (int t = 0; t < CPL; t++) facc[t] = 0.0f;
        int nonempty = 0;
        int j = q;
        uint32_t idn[4];  // the first row ids of the next outer list, fetched one list ahead
        {
            const uint2 m = j < npiece ? smeta[j] : make_uint2(0u, 0u);
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const uint32_t i = (uint32_t)(r * LPR + sub);
                idn[r] = i < (m.y & 0xFFu) ? (uint32_t)indices1[(uint64_t)m.x + i] : 0u;
            }
        }
        for (; __ballot(j < npiece) != 0; j += G2) {
            const uint2 m = j < npiece ? smeta[j] : make_uint2(0u, 0u);
            const int n1 = (int)(m.y & 0xFFu);           // rows of this piece
            const int whole = (int)((m.y >> 8) & 0xFFu);  // rows of the list it belongs to
#pragma unroll
            for (int r = 0; r < 4; r++) sidx[r * LPR + sub] = idn[r];
            wave_sync();
            {
                const int jn = j + G2;
                const uint2 mx = jn < npiece ? smeta[jn] : make_uint2(0u, 0u);
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const uint32_t i = (uint32_t)(r * LPR + sub);
                    idn[r] = i < (mx.y & 0xFFu) ? (uint32_t)indices1[(uint64_t)mx.x + i] : 0u;
                }
            }
            uint32_t acc[R];
#pragma unroll
            for (int r = 0; r < R; r++) acc[r] = 0u;
            const float inv = whole > 0 ? 1.0f / (float)whole : 0.0f;
            // field sums / |N1(u)| into the running means; the fields start over
#define BF_HOP_FLUSH()                                                                            \
    _Pragma("unroll") for (int c = 0; c < CW; c++)                                                \
        _Pragma("unroll") for (int i = 0; i < W::kN; i++) {                                       \
            _Pragma("unroll") for (int f = 0; f < FPR; f++) {                                     \
                const uint32_t fs = (acc[c * W::kN + i] >> (W::kF * f)) & FMAX;                   \
                facc[c * CPW + i + f * W::kN] = fmaf((float)fs, inv, facc[c * CPW + i + f * W::kN]); \
            }                                                                                     \
            acc[c * W::kN + i] = 0u;                                                              \
            __builtin_amdgcn_sched_barrier(0);                                                    \
        }
            // U rows per step: ids first, then the U row loads together, then the field-parallel
            // adds; slots past the end of the list read a zero row
#define BF_HOP_STEP(CNT)                                                                          \
    for (int k = 0; k < (CNT); k += U) {                                                          \
        uint32_t row[U];                                                                          \
        uint32_t w[U][CW];                                                                        \
        _Pragma("unroll") for (int u = 0; u < U; u++) row[u] = sidx[min(k + u, (CNT) - 1)];       \
        _Pragma("unroll") for (int u = 0; u < U; u++) asm volatile("" : "+v"(row[u]));            \
        _Pragma("unroll") for (int u = 0; u < U; u++) {                                           \
            const uint8_t *src = (k + u < (CNT)) ? codes + (uint64_t)row[u] * rb + coff : zero_row; \
            load_words<CW>(src, w[u]);                                                            \
        }                                                                                         \
        _Pragma("unroll") for (int u = 0; u < U; u++)                                             \
            _Pragma("unroll") for (int c = 0; c < CW; c++)                                        \
                _Pragma("unroll") for (int i = 0; i < W::kN; i++)                                 \
                    acc[c * W::kN + i] += (w[u][c] >> (BITS * i)) & W::kMask;                     \
    }
            {
                const int cnt = chunk_ok ? min(n1, ROUND) : 0;
                BF_HOP_STEP(cnt)
            }
            // lists of more than 4*LPR rows: further rounds of ids, fetched in place
            for (int base = ROUND; __ballot(base < n1) != 0; base += ROUND) {
                wave_sync();  // every lane is done with the parked ids
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const int i = base + r * LPR + sub;
                    sidx[r * LPR + sub] = i < n1 ? (uint32_t)indices1[(uint64_t)m.x + (uint32_t)i] : 0u;
                }
                wave_sync();
                const int cnt = chunk_ok ? max(0, min(n1 - base, ROUND)) : 0;
                BF_HOP_STEP(cnt)
            }
#undef BF_HOP_STEP
            wave_sync();  // the id slots are rewritten by the next entry
            nonempty += (m.y >> 16) != 0u && whole > 0 ? 1 : 0;
            BF_HOP_FLUSH()
#undef BF_HOP_FLUSH
        }
        // the destination's groups add up
        for (int mask = LPR; mask < VL; mask <<= 1) {
#pragma unroll
            for (int t = 0; t < CPL; t++) {
                facc[t] += __shfl_xor(facc[t], mask);
                if (t % 4 == 3) __builtin_amdgcn_sched_barrier(0);  // few exchanges in flight: few registers
            }
            nonempty += __shfl_xor(nonempty, mask);
        }
        const bool badv = (__ballot(bad) & vmask) != 0;
        if (badv && alone && valid && lv == 0) raise_status(status, kStatusListTooLong);
        if (valid && q == 0 && chunk_ok && (alone || !badv)) {
            const float inv2 = n2 > 0 ? 1.0f / (float)n2 : 0.0f;
            const float frac = nonempty == n2 ? 1.0f : (float)nonempty * inv2;
            const bool some = n2 > 0;
            const float nanv = __builtin_nanf("");
            const int col0 = sub * CPL;  // first (bit) column of this lane
            if constexpr (PAIR) {
                float4 *dst = reinterpret_cast<float4 *>(out + v * D + col0 / 2);
#pragma unroll
                for (int t = 0; t < CPL; t += 8) {
                    if ((col0 + t) / 2 >= D) break;
                    const float4 a0 = *reinterpret_cast<const float4 *>(sc + col0 + t);
                    const float4 a1 = *reinterpret_cast<const float4 *>(sc + col0 + t + 4);
                    const float4 b0 = *reinterpret_cast<const float4 *>(mn + col0 + t);
                    const float4 b1 = *reinterpret_cast<const float4 *>(mn + col0 + t + 4);
                    const float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
                    const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
                    float x[8];
#pragma unroll
                    for (int i = 0; i < 8; i++) x[i] = fmaf(a[i], facc[t + i] * inv2, b[i] * frac);
                    float4 val = make_float4(x[0] + x[1], x[2] + x[3], x[4] + x[5], x[6] + x[7]);
                    if (!some) val = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (badv) val = make_float4(nanv, nanv, nanv, nanv);
                    dst[t / 8] = val;
                    __builtin_amdgcn_sched_barrier(0);  // one granule's parameters in registers at a time
                }
            } else {
                float4 *dst = reinterpret_cast<float4 *>(out + v * D + col0);
#pragma unroll
                for (int t = 0; t < CPL; t += 4) {
                    if (col0 + t >= D) break;
                    const float4 a = *reinterpret_cast<const float4 *>(sc + col0 + t);
                    const float4 b = *reinterpret_cast<const float4 *>(mn + col0 + t);
                    float4 val;
                    val.x = fmaf(a.x, facc[t] * inv2, b.x * frac);
                    val.y = fmaf(a.y, facc[t + 1] * inv2, b.y * frac);
                    val.z = fmaf(a.z, facc[t + 2] * inv2, b.z * frac);
                    val.w = fmaf(a.w, facc[t + 3] * inv2, b.w * frac);
                    if (!some) val = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (badv) val = make_float4(nanv, nanv, nanv, nanv);
                    dst[t / 4] = val;
                    __builtin_amdgcn_sched_barrier(0);  // one granule's parameters in registers at a time
                }
            }
        }
        wave_sync();  // smeta is rewritten by the next tile
    }
}

template <int BITS, bool WIDE, bool PAIR, bool SPLIT = false>
bool launch_hop_bits(bifeat_params *p, const HopCall &c, int thr, bool alone, const float *mn, const float *sc) {
    using W = LeanSwar<BITS, WIDE>;
    static_assert(!SPLIT || kHopPiece <= W::kCap, "a field holds a piece");
    if (thr > (SPLIT ? 2 * kHopPiece : W::kCap)) return false;
    const int64_t payload = p->payload;
    // words per lane: at most 32 columns per lane stay in registers as fp32 accumulators
    const int cw_max = PAIR ? 1 : (BITS == 8 ? 4 : BITS);
    int cw = 0;
    double best_eff = -1.0;
    for (int cand = cw_max; cand >= 1; cand--) {
        if (payload % (4 * cand)) continue;
        const int chunks = (int)(payload / (4 * cand));
        if (chunks > 64) continue;
        const double eff = (double)chunks / pow2ceil(chunks);
        if (eff > best_eff + 1e-9) {
            best_eff = eff;
            cw = cand;
        }
    }
    if (!cw) return false;
    const int chunks = (int)(payload / (4 * cw));
    const int lpr = pow2ceil(chunks), lpr_log2 = ilog2(lpr);
    // groups per destination: about one per seed-list entry, between 16 and 64 lanes in all
    const int64_t avg2 = c.V2 > 0 ? c.E2 / c.V2 : 1;
    int g2 = 1;
    while (2 * g2 <= avg2 && 2 * g2 * lpr <= 64) g2 *= 2;
    while (g2 * lpr < 16) g2 *= 2;
    const int vpw = 64 / (g2 * lpr);
    const int64_t tiles = (c.V2 + vpw - 1) / vpw;
    const int64_t cap = p->opt_mean_blocks > 0 ? p->opt_mean_blocks : (1 << 16);
    // heavy-first order pays when a wave serves a single destination (measured: 7-15 % there,
    // a loss with two or more per wave); the threshold is the average seed-list length
    const int heavy = BF_HOP_SPLIT && vpw == 1 && avg2 >= 2 ? (int)(avg2 < thr ? avg2 : thr) : 0;
    const int64_t want = ((heavy ? 2 : 1) * tiles + kHopWaves - 1) / kHopWaves;
    const int blocks = (int)(want < cap ? (want < 1 ? 1 : want) : cap);
    const int D = (int)p->D, Dp = PAIR ? 2 * D : D;
    const size_t shm = sizeof(uint32_t) * (size_t)kHopWaves * kHopIds +
                       sizeof(uint2) * (size_t)kHopWaves * vpw * (SPLIT ? 2 * thr : thr);
#define BF_HK(CWV)                                                                                 \
    gather_mean_2hop_lean_kernel<BITS, CWV, WIDE, PAIR, SPLIT><<<blocks, kHopThreads, shm, c.s>>>( \
        c.codes, (uint32_t)p->rb, c.indptr1, c.indices1, c.indptr2, c.indices2, c.V2, D, Dp, mn, sc, \
        p->d_zero, c.out, lpr_log2, ilog2(g2), chunks, thr, heavy, alone ? 1 : 0, c.status)
    if constexpr (PAIR) {
        BF_HK(1);
    } else if constexpr (BITS == 1) {
        BF_HK(1);
    } else if constexpr (BITS == 2) {
        if (cw == 2) BF_HK(2);
        else BF_HK(1);
    } else {
        switch (cw) {
            case 4: BF_HK(4); break;
            case 3: BF_HK(3); break;
            case 2: BF_HK(2); break;
            default: BF_HK(1); break;
        }
    }
#undef BF_HK
    return true;
}

}  // namespace

int hop_lean_max_list() { return 64; }

// The register-accumulator form for affine codes (uniform, 1-bit logarithmic; pair = 2-bit
// logarithmic codes as two bit planes) under the caller's bound `thr` on every list length;
// returns false (nothing launched) when the table's shape is outside what it handles.
bool launch_gather_mean_2hop_lean(bifeat_params *p, const HopCall &c, int thr, bool pair, bool alone) {
    const float *mn = p->d_min, *sc = p->d_scale;
    if (pair) {
        return thr > LeanSwar<1, false>::kCap ? launch_hop_bits<1, true, true>(p, c, thr, alone, mn, sc)
                                              : launch_hop_bits<1, false, true>(p, c, thr, alone, mn, sc);
    }
    switch (p->scheme.bits) {
        case 1:
            return thr > LeanSwar<1, false>::kCap ? launch_hop_bits<1, true, false>(p, c, thr, alone, mn, sc)
                                                  : launch_hop_bits<1, false, false>(p, c, thr, alone, mn, sc);
        case 2: return launch_hop_bits<2, false, false>(p, c, thr, alone, mn, sc);
        case 4:
            if (thr <= LeanSwar<4, false>::kCap) return launch_hop_bits<4, false, false>(p, c, thr, alone, mn, sc);
            if (thr <= 2 * kHopPiece && BF_HOP_SPLIT16) return launch_hop_bits<4, false, false, true>(p, c, thr, alone, mn, sc);
            return launch_hop_bits<4, true, false>(p, c, thr, alone, mn, sc);
        default: return launch_hop_bits<8, false, false>(p, c, thr, alone, mn, sc);
    }
}

}  // namespace bf
