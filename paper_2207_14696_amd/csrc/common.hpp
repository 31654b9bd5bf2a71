// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <vector>

#include "bifeat.h"

// Quantizer state behind the opaque bifeat_params handle.
struct bifeat_params {
    bifeat_scheme scheme{};
    int64_t D = 0;
    int64_t ncodes = 0;  // codes per row: D, or P for vector codes
    int64_t rb = 0;      // bytes from one packed row to the next, multiple of 16
    int64_t payload = 0; // bytes of a row that hold codes, rounded up to 16 (rb >= payload; the
                         // rest is zero padding of a line-aligned table, option "row_align")
    int P = 0;           // vector codes: number of parts
    int cbytes = 1;      // vector codes: bytes per stored index (2 beyond 256 entries)

    // host copies (valid when host_valid)
    std::vector<float> h_min, h_max, h_scale, h_inv;  // uniform, [D] each
    double e_min = 0.0, e_max = 0.0;                  // log
    std::vector<float> h_T, h_V;                      // log: [H-1], [2^bits]
    std::vector<float> h_cb;                          // vq: [P][len][w]
    std::vector<float> h_rnorm;                       // vq, cosine metric: 1/|entry|, [P][len]
    bool host_valid = false;

    // device block (allocated on first GPU use)
    int device = -1;
    float *d_block = nullptr;
    float *d_min = nullptr, *d_scale = nullptr, *d_inv = nullptr, *d_max = nullptr;
    float *d_T = nullptr, *d_V = nullptr, *d_cb = nullptr;
    float *d_rnorm = nullptr;   // vq, cosine metric: [P][len]
    float *d_train = nullptr;   // vq training scratch: sums [P][len][w], counts [P][len]
    float *d_dist = nullptr;    // vq training: summed squared distance per Lloyd round (64 slots)
    uint8_t *d_scratch = nullptr;  // grow-only workspace (vector codes: slice-major code strips)
    size_t scratch_bytes = 0;
    std::vector<void *> retired;   // outgrown workspaces, kept allocated until the handle dies
    uint8_t *d_zero = nullptr;  // 64 zero bytes (stand-in row for masked loads)
    int32_t *d_fit = nullptr;  // uniform: ordered-int keys [min D | max D]; log: bits of [mmin, mmax]
    unsigned long long *d_hist = nullptr;  // log, clipped fit: digit histograms [2][kLogHistBins]

    // log scheme, clipped fit: three radix-selection passes over the data
    double clip_fraction = 0.0;  // 0 = plain fit of the extreme magnitudes
    int fit_pass = 0;
    uint32_t clip_prefix[2] = {0, 0};      // digits fixed so far for the low / high rank
    unsigned long long clip_rank[2] = {0, 0};  // rank still to find inside that prefix

    bool fitted = false;
    bool fit_open = false;
    int64_t fit_rows = 0;
    bool vq_seeded = false;     // codebooks initialised from a sample chunk
    int64_t vq_last_rows = 0;   // rows of the last training chunk
    int vq_last_rounds = 0;

    // status word the kernels can raise without the host waiting for them: pinned host memory
    // mapped into the device's address space (h_status / d_status name the same word)
    int32_t *h_status = nullptr;
    int32_t *d_status = nullptr;

    // launch tuning (0 = automatic)
    int opt_mean_slots = 0;
    int opt_mean_blocks = 0;
    int opt_max_blocks = 0;    // cap on workgroups of the gather kernels
    int opt_mean_lean = 1;        // 0: never use the short-list kernel
    int opt_mean_max_degree = 0;  // caller's promise: no neighbour list is longer (0 = unknown)
    int opt_vq_iters = 10;        // Lloyd rounds per training chunk
    int opt_vq_sliced = 1;        // 0: vector codes decode from L2 instead of LDS-resident slices
    int opt_dequant_flat = 0;  // 1: gather_dequant without the LDS-staged tile kernel
    int opt_mean_generic = 0;  // 1: route uniform tables through the float-accumulate kernel
    int opt_validate = 0;      // 1: check indices / list bounds on the GPU before every gather (synchronises)
    int opt_row_align = 16;    // 16: rows packed back to back; 128: no row straddles a 128-byte line needlessly
};

namespace bf {

constexpr int kThreads = 256;
constexpr int kLogHistBins = 2048;  // 11-bit digits of the clipped log fit
// number of workgroups that fills the chip a few times over: 256 CUs x 8
constexpr int kMaxBlocks = 2048;

hipError_t launch_fit_reset(bifeat_params *p, hipStream_t s);
hipError_t launch_fit_update(bifeat_params *p, const void *chunk, int dtype, int64_t rows,
                             hipStream_t s);
hipError_t launch_finalize_uniform(bifeat_params *p, hipStream_t s);
void launch_log_hist_reset(bifeat_params *p, hipStream_t s);
hipError_t launch_log_hist_update(bifeat_params *p, const void *chunk, int dtype, int64_t rows,
                                  hipStream_t s);
hipError_t launch_vq_train(bifeat_params *p, const void *chunk, int dtype, int64_t rows, bool init,
                           int rounds, hipStream_t s);
hipError_t launch_quantize(bifeat_params *p, const void *chunk, int dtype, int64_t rows,
                           uint8_t *codes_row0, hipStream_t s);
hipError_t launch_gather_codes(bifeat_params *p, const uint8_t *codes, const int64_t *idx,
                               int64_t M, uint8_t *out, hipStream_t s);
// planes: workspace for the vector-code kernels (nullptr = the handle's own, grown as needed)
hipError_t launch_gather_dequant(bifeat_params *p, const uint8_t *codes, const int64_t *idx,
                                 int64_t M, float *out, hipStream_t s, uint32_t *planes = nullptr);
// One fused gather + aggregate request as the launchers of the mean kernels see it.
struct MeanCall {
    const uint8_t *codes;   // packed table
    int64_t N;              // its rows
    const int64_t *indptr;  // [V + 1]
    const void *indices;    // [E] row ids, int64 or (idx32) int32
    bool idx32;
    int64_t V, E;
    float *out;             // [V x D]
    int agg_sum;            // 1: sum aggregator (no division by the list length)
    // the caller's promise that no list is longer (0 = none given).  A kernel that relies on
    // it (no complementary pass for longer lists is launched) writes a row of NaNs for a list
    // that breaks it and raises kStatusListTooLong in *status
    int max_degree;
    int32_t *status;
    hipStream_t s;
};
constexpr int32_t kStatusListTooLong = 1;

hipError_t launch_gather_mean(bifeat_params *p, const MeanCall &c);
// min_len: lists with at most this many neighbours are skipped (left to the
// short-list kernel); -1 = none
void launch_gather_mean_swar(bifeat_params *p, const MeanCall &c, int vec, int min_len);
// grow-only library workspace (p->d_scratch); false if the allocation fails or `s` is being
// captured into a graph (nothing is allocated during a capture)
bool ensure_scratch(bifeat_params *p, size_t bytes, hipStream_t s);
// bytes of workspace a vector-code gather of M requested rows needs
size_t vq_gather_scratch_bytes(const bifeat_params *p, int64_t M);
// the library's fixed per-GPU workspace (a static device array): its size, and its address
// on the current device
size_t static_scratch_bytes();
hipError_t static_scratch_ptr(uint8_t **out);
// 1/|entry| for every codebook entry, fp64 inside (cosine metric)
void launch_vq_rnorm(bifeat_params *p, hipStream_t s);
// nearest-entry search of `rows` rows into codes_row0 (row stride rb bytes, indices of
// `cbytes` bytes; bytes from P*cbytes to rb are zeroed)
template <typename T>
void launch_vq_assign(bifeat_params *p, const T *x, int64_t rows, uint8_t *codes_row0, int64_t rb,
                      hipStream_t s);
// counts violations of 0 <= idx[i] < N (and, with indptr, of indptr[0] == 0, indptr
// non-decreasing, indptr[V] == E, no list longer than max_len if that is positive) into
// *d_bad (zeroed first)
void launch_validate(const int64_t *idx, int64_t M, int64_t N, const int64_t *indptr, int64_t V,
                     int64_t E, int64_t max_len, int32_t *d_bad, hipStream_t s);
// fp32-row neighbourhood mean / sum (layers after the first) and the sum of row lengths
hipError_t launch_aggregate_rows(const float *x, int64_t D, const int64_t *indptr,
                                 const int64_t *indices, int64_t V, int64_t E, int sum, float *out,
                                 hipStream_t s);
hipError_t launch_row_length_sum(const float *h, int64_t n, int64_t D, double *acc, hipStream_t s);
void launch_zero_doubles(double *p, int n, hipStream_t s);
bool launch_gather_dequant_vq_sliced(bifeat_params *p, const uint8_t *codes, const int64_t *idx,
                                     int64_t M, float *out, hipStream_t s, uint32_t *planes);
bool launch_gather_mean_vq_sliced(bifeat_params *p, const MeanCall &c);
int lean_capacity(int bits, bool wide);
// logarithmic codes of 4 / 8 bits, lists of at most logf_capacity() neighbours
int logf_capacity();
// The short-list kernels: lists of more than `lo` and at most `thr` rows; alone = no other
// kernel is launched for the longer lists (they then get NaN rows and raise the status word).
// Each returns false (nothing launched) when the table's shape is outside what it handles.
bool launch_gather_mean_logf(bifeat_params *p, const MeanCall &c, int thr, bool alone);
bool launch_gather_mean_lean_log2(bifeat_params *p, const MeanCall &c, int thr, bool wide, int lo,
                                  bool alone);
bool launch_gather_mean_lean(bifeat_params *p, const MeanCall &c, int thr, bool wide, int lo,
                             bool alone);

// Two rounds of the neighbourhood mean from the packed table: the outer block's lists hold
// table rows (one list per first-round destination), the seed block's lists hold first-round
// destinations.
struct HopCall {
    const uint8_t *codes;
    int64_t N;
    const int64_t *indptr1, *indices1;  // [V1 + 1], [E1]
    int64_t V1, E1;
    const int64_t *indptr2, *indices2;  // [V2 + 1], [E2], entries in [0, V1)
    int64_t V2, E2;
    float *out;      // [V2 x D]
    int max_degree;  // the caller's bound on every list length of both blocks (0 = none given)
    int32_t *status;
    hipStream_t s;
};
hipError_t launch_gather_mean_2hop(bifeat_params *p, const HopCall &c);
// alone: no other kernel takes the destinations with a list longer than thr (they get NaN rows
// and raise the status word); otherwise they are left unwritten for the general kernel
bool launch_gather_mean_2hop_lean(bifeat_params *p, const HopCall &c, int thr, bool pair, bool alone);
int hop_lean_max_list();
bool launch_gather_mean_2hop_vq_sliced(bifeat_params *p, const HopCall &c);

// ---- order-preserving float <-> int keys for atomic min/max
__host__ __device__ inline int32_t float_key(float f) {
    union { float f; int32_t i; } u;
    u.f = f;
    return u.i >= 0 ? u.i : (u.i ^ 0x7FFFFFFF);
}
__host__ __device__ inline float key_float(int32_t k) {
    union { float f; int32_t i; } u;
    u.i = k >= 0 ? k : (k ^ 0x7FFFFFFF);
    return u.f;
}
constexpr int32_t kKeyPosInf = 0x7F800000;
constexpr int32_t kKeyNegInf = (int32_t)0x807FFFFFu;

// ---- 4 consecutive elements of a row as floats
__device__ inline float4 load4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ inline float4 load4(const __half *p) {
    uint2 u = *reinterpret_cast<const uint2 *>(p);
    __half2 a = *reinterpret_cast<__half2 *>(&u.x);
    __half2 b = *reinterpret_cast<__half2 *>(&u.y);
    float2 fa = __half22float2(a), fb = __half22float2(b);
    return make_float4(fa.x, fa.y, fb.x, fb.y);
}
// Output rows are written once and not read again by these kernels: streaming
// (non-temporal) stores keep them from evicting the packed table from the
// caches the gathers depend on.
__device__ inline void store_stream(float4 *p, const float4 v) {
#ifdef BF_PLAIN_STORE
    *p = v;
    return;
#endif
    __builtin_nontemporal_store(v.x, &p->x);
    __builtin_nontemporal_store(v.y, &p->y);
    __builtin_nontemporal_store(v.z, &p->z);
    __builtin_nontemporal_store(v.w, &p->w);
}
__device__ inline void store_stream(uint4 *p, const uint4 v) {
    __builtin_nontemporal_store(v.x, &p->x);
    __builtin_nontemporal_store(v.y, &p->y);
    __builtin_nontemporal_store(v.z, &p->z);
    __builtin_nontemporal_store(v.w, &p->w);
}
// index arrays are streamed once as well
template <typename T>
__device__ inline T load_stream(const T *p) { return __builtin_nontemporal_load(p); }

__device__ inline float load1(const float *p) { return *p; }
__device__ inline float load1(const __half *p) { return __half2float(*p); }

// ---- helpers shared by the tile kernels
// orders a wave's LDS writes before its later LDS reads (all lanes of a wave execute each DS
// instruction together, in program order): no workgroup barrier needed inside a wave's tile
__device__ inline void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

struct __attribute__((aligned(4))) U3 { uint32_t x, y, z; };

// CW consecutive 32-bit words of a packed row with one load instruction
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

// ---- field-parallel integer sums of packed code words (the short-list aggregation kernels)
template <int BITS, bool WIDE> struct LeanSwar;
// kF: field width, kN: registers per 32-bit word; register i, field f holds the
// sum of code number i + f*kN; kCap = rows a field can sum.  The WIDE forms
// spend more shift+mask work per word on fields that hold longer lists.
template <bool WIDE> struct LeanSwar<8, WIDE> { static constexpr int kF = 16, kN = 2, kCap = 257; static constexpr uint32_t kMask = 0x00FF00FFu; };
template <> struct LeanSwar<4, false> { static constexpr int kF = 8, kN = 2, kCap = 17; static constexpr uint32_t kMask = 0x0F0F0F0Fu; };
template <> struct LeanSwar<4, true> { static constexpr int kF = 16, kN = 4, kCap = 4369; static constexpr uint32_t kMask = 0x000F000Fu; };
template <bool WIDE> struct LeanSwar<2, WIDE> { static constexpr int kF = 8, kN = 4, kCap = 85; static constexpr uint32_t kMask = 0x03030303u; };
template <> struct LeanSwar<1, false> { static constexpr int kF = 4, kN = 4, kCap = 15; static constexpr uint32_t kMask = 0x11111111u; };
template <> struct LeanSwar<1, true> { static constexpr int kF = 8, kN = 8, kCap = 255; static constexpr uint32_t kMask = 0x01010101u; };

// a kernel reports a broken caller promise: a plain system-scope store of the code into the
// mapped status word (no read-modify-write across the bus; the word holds the last code raised)
__device__ inline void raise_status(int32_t *status, int32_t code) {
    __hip_atomic_store(status, code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

inline int pow2ceil(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}
inline int ilog2(int x) {
    int l = 0;
    while ((1 << l) < x) l++;
    return l;
}

inline int blocks_for(int64_t threads_needed, int64_t cap = kMaxBlocks) {
    int64_t b = (threads_needed + kThreads - 1) / kThreads;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (int)b;
}

}  // namespace bf
