// Fused gather + decode + neighbourhood mean for logarithmic codes of 4 and 8 bits
// (Sec. 3.1 Eq. (2) decode, Appendix A.1 mean), short lists.
//
// Their decode is a table of 16 or 256 values, not an affine map, so the integer-sum
// kernels of the other scalar codes do not apply: every code is looked up and added in
// fp32.  The shape is that of the short-list kernel of the uniform codes: a wave takes
// 64 / LPR consecutive destinations, LPR lanes per destination each owning 16 bytes of
// the packed row (one 16-byte load per neighbour and lane, kLogfU neighbours in
// flight), the decode table in LDS (a 16-entry table is conflict-free: lanes that hit
// the same bank read the same word), and the tile's output rows leave as one contiguous
// run of streaming 16-byte stores after a transposition through LDS.
#include "common.hpp"

namespace bf {
namespace {

constexpr int kLogfWaves = kThreads / 64;
constexpr int kLogfU = 3;  // neighbour rows in flight per lane (2: 7 % slower, 4: no faster)

// IT: the type of a list entry (int64_t or int32_t).  alone: no other kernel takes the lists
// longer than thr: such a list gets a row of NaNs and raises the status word.
template <int BITS, typename IT>
__global__ __launch_bounds__(kThreads) void gather_mean_logf_kernel(
    const uint8_t *__restrict__ codes, uint32_t rb, const int64_t *__restrict__ indptr,
    const IT *__restrict__ indices, int64_t V, int D, const float *__restrict__ table,
    float *__restrict__ out, int lpr_log2, int chunks, int thr, int agg_sum, int alone,
    int32_t *__restrict__ status) {
    constexpr int CPW = 32 / BITS;    // codes per 32-bit word
    constexpr int CPL = 4 * CPW;      // columns per lane (16 bytes of codes)
    constexpr int NS = CPL / 4;       // 16-byte slots of decoded values per lane
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    // a wave's stage: 64 lanes x CPL floats, rows of LPR * CPL floats per destination
    __shared__ float s_table[1 << BITS];
    __shared__ __attribute__((aligned(16))) float s_stage[kLogfWaves][64 * CPL];
    __shared__ float s_meta[kLogfWaves][64];
    for (int i = threadIdx.x; i < (1 << BITS); i += kThreads) s_table[i] = table[i];
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *stage = s_stage[wave];
    float *meta = s_meta[wave];
    const int LPR = 1 << lpr_log2;
    const int dpw_log2 = 6 - lpr_log2, dpw = 1 << dpw_log2;
    const int lane_chunk = lane & (LPR - 1), d_local = lane >> lpr_log2;
    const bool chunk_ok = lane_chunk < chunks;
    const uint32_t coff = (uint32_t)lane_chunk * 16u;
    const int nf4 = D >> 2;
    const int step_d = 64 / nf4, step_f = 64 % nf4;
    const int lane_d = lane / nf4, lane_f = lane % nf4;
    const int64_t tiles = (V + dpw - 1) >> dpw_log2;
    const int64_t n_waves = (int64_t)gridDim.x * kLogfWaves;
    // slot s of a lane's decoded values is parked at slot s ^ swz of its stage piece, so
    // that the lanes of a destination, whose pieces are CPL floats apart, spread over
    // the banks instead of all hitting the same four
    const int swz = lane_chunk & (NS - 1);

    for (int64_t tile = (int64_t)blockIdx.x * kLogfWaves + wave; tile < tiles; tile += n_waves) {
        const int64_t v_tile = tile << dpw_log2;
        const int ndst = (int)min((int64_t)dpw, V - v_tile);
        int64_t beg = 0, end = 0;
        if (d_local < ndst) {
            beg = indptr[v_tile + d_local];
            end = indptr[v_tile + d_local + 1];
        }
        const int64_t n64 = end - beg;
        const bool mine = d_local < ndst && n64 <= thr;  // longer lists: the general kernel
        const bool over = alone && d_local < ndst && n64 > thr;  // a broken promise
        if (__ballot(mine || over) == 0) continue;       // nothing for this launch in the tile
        const int n = mine ? (int)n64 : 0;
        if (lane_chunk == 0) {
            meta[d_local] = mine ? (n > 0 ? (agg_sum ? 1.0f : 1.0f / (float)n) : 0.0f)
                                 : (over ? __builtin_nanf("") : -1.0f);
            if (over) raise_status(status, kStatusListTooLong);
        }

        float acc[CPL];
#pragma unroll
        for (int j = 0; j < CPL; j++) acc[j] = 0.0f;
        const IT *ip = indices + beg;
        const int cnt = chunk_ok ? n : 0;
        for (int k = 0; k < cnt; k += kLogfU) {
            IT row[kLogfU];
            uint4 w[kLogfU];
#pragma unroll
            for (int u = 0; u < kLogfU; u++) row[u] = ip[min(k + u, cnt - 1)];
            // the index loads stay together and unconditional, the row loads right behind
#pragma unroll
            for (int u = 0; u < kLogfU; u++) asm volatile("" : "+v"(row[u]));
#pragma unroll
            for (int u = 0; u < kLogfU; u++)
                w[u] = *reinterpret_cast<const uint4 *>(codes + (uint64_t)row[u] * rb + coff);
#pragma unroll
            for (int u = 0; u < kLogfU; u++) {
                if (k + u < cnt) {  // past the list's end the last row is re-read and not added
                    const uint32_t word[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
#pragma unroll
                    for (int c = 0; c < 4; c++)
#pragma unroll
                        for (int i = 0; i < CPW; i++)
                            acc[c * CPW + i] += s_table[(word[c] >> (BITS * i)) & MASK];
                }
            }
        }
        {
            float4 *sp = reinterpret_cast<float4 *>(stage + lane * CPL);
#pragma unroll
            for (int s = 0; s < NS; s++)
                sp[s ^ swz] = make_float4(acc[4 * s], acc[4 * s + 1], acc[4 * s + 2], acc[4 * s + 3]);
        }
        wave_sync();

        // ---- the tile's output rows, one contiguous span of ndst * nf4 float4 granules
        float4 *span = reinterpret_cast<float4 *>(out + v_tile * D);
        const int ngran = ndst * nf4;
        int d = lane_d, f = lane_f;
        for (int m = lane; m < ngran; m += 64) {
            const float md = meta[d];
            const int col = 4 * f;
            const int owner = col / CPL, slot = (col % CPL) >> 2;
            const float4 q = *reinterpret_cast<const float4 *>(
                stage + ((d << lpr_log2) + owner) * CPL + 4 * (slot ^ (owner & (NS - 1))));
            const bool some = md > 0.0f;  // md == 0: empty list, zero row
            float4 val = make_float4(some ? q.x * md : 0.0f, some ? q.y * md : 0.0f,
                                     some ? q.z * md : 0.0f, some ? q.w * md : 0.0f);
            if (md != md) val.x = val.y = val.z = val.w = md;  // list beyond the promised bound
            if (!(md < 0.0f)) store_stream(&span[m], val);  // md < 0: not this kernel's destination
            d += step_d;
            f += step_f;
            if (f >= nf4) {
                f -= nf4;
                d++;
            }
        }
        wave_sync();  // the stage is rewritten by the next tile
    }
}

}  // namespace

// Lists of more than this many neighbours stay with the general kernel (fp32 sums of at
// most 64 terms keep the rounding error below 4e-6 of the largest decodable magnitude).
int logf_capacity() { return 64; }

// False (nothing launched) when the shape is outside what the kernel handles.
bool launch_gather_mean_logf(bifeat_params *p, const MeanCall &c, int thr, bool alone) {
    const int bits = p->scheme.bits;
    const int64_t c16 = p->payload / 16;  // lanes that fetch a row (its stride is p->rb)
    if ((bits != 4 && bits != 8) || p->D % 4 || (uintptr_t)c.out % 16 || (uintptr_t)c.codes % 16 ||
        c16 > 64 || c.V <= 0)
        return false;
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < c16) lpr_log2++;
    const int dpw = 64 >> lpr_log2;
    const int64_t tiles = (c.V + dpw - 1) / dpw;
    const int64_t want = (tiles + kLogfWaves - 1) / kLogfWaves;
    const int64_t cap = p->opt_mean_blocks > 0 ? p->opt_mean_blocks : (1 << 16);
    const int blocks = (int)(want < cap ? want : cap);
#define BF_LF(B, IT)                                                                              \
    gather_mean_logf_kernel<B, IT><<<blocks, kThreads, 0, c.s>>>(                                 \
        c.codes, (uint32_t)p->rb, c.indptr, (const IT *)c.indices, c.V, (int)p->D, p->d_V, c.out, \
        lpr_log2, (int)c16, thr, c.agg_sum, alone ? 1 : 0, c.status)
    if (bits == 4) {
        if (c.idx32) BF_LF(4, int32_t);
        else BF_LF(4, int64_t);
    } else {
        if (c.idx32) BF_LF(8, int32_t);
        else BF_LF(8, int64_t);
    }
#undef BF_LF
    return true;
}

}  // namespace bf
