/*
 * bifeat.h - C ABI of the MI355X feature-loading library for BiFeat
 * (graph feature quantization, arXiv 2207.14696).
 *
 * The library keeps a node-feature table in compressed form in GPU memory and
 * serves minibatch iterations from it:
 *   - one-time preprocessing (paper Sec. 3.3: done once, ahead of training): fit the
 *     quantizer to the table, chunk by chunk, then encode + pack each chunk;
 *   - per iteration (Sec. 3.3): gather the compressed rows of the sampled
 *     nodes and decode them to fp32, optionally fused with the first layer's
 *     neighbourhood mean (Appendix A.1, g_i = 1/|N(i)| sum_{j in N(i)} g_j).
 *
 * Conventions, all entry points
 *   - Every data pointer documented as DEVICE points to GPU memory owned by
 *     the caller; HOST pointers are ordinary host memory.  The library keeps no
 *     reference to caller memory after a call returns, except that work
 *     enqueued on `stream` reads/writes the DEVICE buffers until it completes.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return without synchronising unless stated.
 *   - Return value: BIFEAT_OK (0) or a negative bifeat_status.  Argument
 *     errors are detected before any GPU call is made.  bifeat_strerror()
 *     gives a description (for BIFEAT_EHIP: the HIP error text of the last
 *     failure on the calling thread).
 *   - Calls on one bifeat_params handle must not overlap in time (they share
 *     its fit state and, for vector codes, its workspace: the transposed
 *     codes of the rows a call requests).  Different handles are independent.
 *   - The per-iteration calls (gather_codes / gather_dequant / gather_mean /
 *     gather_sum) only enqueue kernels: no memset, no synchronisation, and no
 *     allocation except growth of the vector-code workspace when a request is
 *     larger than any before (bifeat_reserve sizes it ahead of time).  An
 *     outgrown workspace stays allocated until the handle is destroyed, so
 *     work in flight and HIP graphs captured from earlier calls keep valid
 *     addresses.  The calls can be captured into a HIP graph (with option
 *     "validate" off); nothing is allocated while the stream is capturing: a
 *     vector-code request larger than the workspace is then decoded by the
 *     slower kernels that need none.
 *   - Row indices must satisfy 0 <= idx < N, indptr must be non-decreasing with
 *     indptr[0] = 0 and indptr[V] = E; this is the caller's contract and is not
 *     checked on the GPU - unless option "validate" = 1 is set: every gather
 *     call then first checks it (and, for gather_mean / gather_sum, a bound
 *     promised through option "mean_max_degree") with a small kernel,
 *     synchronises `stream`, and returns BIFEAT_EINVAL without launching the
 *     gather when it is broken.
 *   - Packed layout (the paper fixes none; Appendix C only advises against
 *     elaborate bit packing): row-major; scalar codes: column j's `bits`-bit
 *     code at bit (j*bits) mod 8 of byte floor(j*bits/8), column 0 in the
 *     least significant bits; vector codes: byte p = codebook index of part p
 *     (codebooks of more than 256 entries: bytes 2p, 2p+1 = the index, low
 *     byte first - the whole-byte alignment of Appendix C);
 *     row stride bifeat_row_bytes() = payload rounded up to 16 bytes, pad = 0.
 *     With option "row_align" = 128 (set it before the table is sized and packed)
 *     the stride is instead the next power of two for payloads of up to 128
 *     bytes and the next multiple of 128 above that, pad = 0: a gathered row
 *     then never touches more 128-byte memory lines than its length requires
 *     (a 96-byte row, e.g. 768 one-bit codes or 96 one-byte indices, costs one
 *     line instead of 1.5 on average, for a table one third larger).
 */
#ifndef BIFEAT_H
#define BIFEAT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    /* bifeat_fit_finalize only: the fit needs another pass over the same data -
     * call bifeat_fit_update for every chunk again, then finalize again */
    BIFEAT_FIT_AGAIN = 1,
    BIFEAT_OK = 0,
    BIFEAT_EINVAL = -1,  /* bad argument (null pointer, unsupported bits, size <= 0, ...) */
    BIFEAT_ENOTFIT = -2, /* quantizer parameters not fitted / set yet */
    BIFEAT_EHIP = -3,    /* a HIP runtime call or kernel launch failed */
    BIFEAT_ENOTSUP = -4, /* valid request this build does not implement */
    BIFEAT_ELIMIT = -5   /* request larger than a fixed limit (bifeat_gather_dequant_static) */
} bifeat_status;

typedef enum {
    /* evenly spaced levels between per-column min and max - the ordinary
     * uniform quantization that Sec. 3.1 starts from */
    BIFEAT_SQ_UNIFORM = 0,
    /* BiFeat-SQ: sign-split uniform quantization of clipped log2|x|,
     * Sec. 3.1 Eq. (1), decoded by Eq. (2) */
    BIFEAT_SQ_LOG = 1,
    /* BiFeat-VQ: per-part codebooks, Sec. 3.2 */
    BIFEAT_VQ = 2
} bifeat_kind;

typedef enum { BIFEAT_F32 = 0, BIFEAT_F16 = 1 } bifeat_dtype;

/* Sec. 3.2 allows two rules for the nearest codebook entry: Euclidean distance
 * or cosine similarity.  Cosine: the entry with the largest (x . C_c)/|C_c| (the
 * part's own norm is a common positive factor and is left out; an all-zero part
 * or entry scores 0); entries stay arithmetic means of their members and decode
 * returns the entry unchanged. */
typedef enum { BIFEAT_VQ_L2 = 0, BIFEAT_VQ_COSINE = 1 } bifeat_vq_metric;

typedef struct {
    int32_t kind;      /* bifeat_kind */
    int32_t bits;      /* scalar kinds: 1, 2, 4 or 8 bits per value */
    int32_t vq_width;  /* BIFEAT_VQ: dims per part (1..128); P = ceil(D/width) parts, a short
                          last part is zero-padded */
    int32_t vq_length; /* BIFEAT_VQ: entries per codebook: 2..256 stored as one byte per
                          part, 257..16384 as two (Appendix C) */
    int32_t vq_metric; /* BIFEAT_VQ: bifeat_vq_metric */
} bifeat_scheme;

/* Opaque quantizer state: scheme, D, fitted parameters (host + device copies).
 * Device memory is allocated on first GPU use, on the device current then, and
 * released by bifeat_params_destroy. */
typedef struct bifeat_params bifeat_params;

int bifeat_params_create(const bifeat_scheme *scheme, int64_t D, bifeat_params **out);
void bifeat_params_destroy(bifeat_params *p);

/* Packed bytes per row (a multiple of 16), or BIFEAT_EINVAL. */
int64_t bifeat_row_bytes(const bifeat_params *p);
/* Codes per row: D (scalar kinds) or the number of parts (BIFEAT_VQ). */
int64_t bifeat_codes_per_row(const bifeat_params *p);

/* ---- fitting (Sec. 3.1: e_min/e_max bound log2|x| once outliers are clipped;
 *      uniform: per-column range).  Streaming: reset, update per chunk, finalize.
 * chunk: DEVICE, [rows x D] row-major, `dtype` elements.
 * SQ_UNIFORM: per-column min and max over all chunks (NaNs skipped, a zero
 *   result stored as +0); finalize derives, per column, in fp64 rounded once
 *   to fp32: scale = (max-min)/L, inv = L/(max-min), L = 2^bits-1 (both 0 for a
 *   constant column).  Runs entirely on `stream`.
 * SQ_LOG: smallest nonzero and largest finite |x| over all chunks; finalize
 *   sets e_min/e_max to their log2 and builds the tables of
 *   bifeat_params_set_log.  finalize synchronises `stream` (the two
 *   magnitudes come back to the host, where log2/exp2 are evaluated in fp64).
 *   With a clip fraction p > 0 (bifeat_fit_set_log_clip) the range ends are
 *   instead the exact order statistics of the n finite nonzero magnitudes at
 *   ranks floor(p (n-1)) and ceil((1-p) (n-1)) (Sec. 3.1 clips outliers before
 *   taking the range; Appendix C leaves the fraction open).  They are found
 *   by radix selection in three passes: finalize returns BIFEAT_FIT_AGAIN
 *   after the first and second pass, and the caller streams the same chunks
 *   through bifeat_fit_update again (a pass over different data ends the fit
 *   with BIFEAT_EINVAL); the third finalize returns BIFEAT_OK.  Each finalize
 *   synchronises `stream`.
 * BIFEAT_VQ (Sec. 3.2 k-means per part; Appendix D: on a uniform row sample,
 *   which is what the caller passes as the chunk): the first chunk after a
 *   reset seeds every part's codebook with the sub-vectors of its first
 *   `vq_length` rows (it must have at least that many); every update then runs
 *   Lloyd rounds over its chunk (10, option "vq_iters"): nearest entry by the
 *   encoder's rule for the scheme's metric, entry = mean of its members, an
 *   entry without members keeps its value.  Sums are accumulated with fp32
 *   atomics, so the codebooks are reproducible in distortion, not bit for bit.
 *   Training a large or cosine codebook uses library scratch (two bytes per
 *   part and sample row).  finalize synchronises `stream` for the cosine metric
 *   (the entry norms are evaluated on the host in fp64).
 * finalize without any update returns BIFEAT_ENOTFIT. */
int bifeat_fit_reset(bifeat_params *p, void *stream);
/* SQ_LOG: clip fraction for the fits that follow, 0 <= fraction < 0.5 (0 = the
 * plain fit of the extreme magnitudes).  Not while a fit is open. */
int bifeat_fit_set_log_clip(bifeat_params *p, double fraction);
int bifeat_fit_update(bifeat_params *p, const void *chunk, int32_t dtype, int64_t rows,
                      void *stream);
int bifeat_fit_finalize(bifeat_params *p, void *stream);

/* ---- setting / reading parameters.  HOST pointers; arrays are copied.
 * set_* uploads synchronously and marks the parameters fitted.
 * get_* synchronises the device; any output pointer may be NULL.
 * uniform: min[D], max[D] in; min, max, scale, inv [D] out.
 * log:     e_min <= e_max in; out also T[2^(bits-1) - 1] (bin edges in |x|,
 *          T_i = exp2(e_min + i*(e_max-e_min)/H), H = 2^(bits-1)) and
 *          V[2^bits] (Eq. (2): V[H+l] = exp2(e_min + (l+.5)*(e_max-e_min)/H),
 *          V[H-1-l] = -V[H+l]).
 * vq:      codebooks [P][length][width] fp32. */
int bifeat_params_set_uniform(bifeat_params *p, const float *mn, const float *mx);
int bifeat_params_get_uniform(bifeat_params *p, float *mn, float *mx, float *scale, float *inv);
int bifeat_params_set_log(bifeat_params *p, double e_min, double e_max);
int bifeat_params_get_log(bifeat_params *p, double *e_min, double *e_max, float *T, float *V);
int bifeat_params_set_codebooks(bifeat_params *p, const float *codebooks);
int bifeat_params_get_codebooks(bifeat_params *p, float *codebooks);
/* BIFEAT_VQ: mean squared Euclidean distance between a part and its assigned
 * entry (summed over parts, either metric) at each Lloyd round's assignment
 * step of the last bifeat_fit_update; out: HOST [n], n <= 64.  Synchronises
 * the device. */
int bifeat_vq_distortion(bifeat_params *p, float *out, int32_t n);

/* ---- encode + pack one chunk (Sec. 3.1 Eq. (1); Sec. 3.2 nearest entry).
 * chunk: DEVICE [rows x D]; codes: DEVICE base of the packed table; rows
 * [row0, row0+rows) of it are written (every byte of each row, padding
 * included).
 * SQ_UNIFORM: q = clamp(rne((x - min_j) * inv_j), 0, L), fp32, each operation
 *   rounded separately; NaN -> 0.
 * SQ_LOG: H = 2^(bits-1), l = #{i : |x| >= T_i}, q = H + l if x > 0 else
 *   H - 1 - l (zero and NaN on the non-positive side, as the text of Sec. 3.1
 *   groups them).
 * BIFEAT_VQ: per part, index of the entry with the smallest squared Euclidean
 *   distance (fp32, dims ascending, multiply and add rounded separately; ties
 *   to the lowest index; a short last part is zero-padded); cosine metric:
 *   the largest fp32 dot product (same accumulation) times
 *   fp32(1/sqrt(sum_d C_cd^2)), sum and root in fp64. */
int bifeat_quantize(bifeat_params *p, const void *chunk, int32_t dtype, int64_t rows,
                    uint8_t *codes, int64_t row0, void *stream);

/* ---- host bookkeeping of include/bifeat_produce.hpp (fit and encode of a table whose values
 * are produced inside the kernels by a caller-defined source; the kernels themselves are C++
 * templates in that header).  fit_begin: what bifeat_fit_update does before its kernel (opens
 * the fit if none is open); BIFEAT_ENOTSUP for vector codes and for a logarithmic fit with a
 * clip fraction.  fit_end: accounts `rows` more fitted rows.  quantize_check: the argument and
 * state checks of bifeat_quantize (BIFEAT_ENOTSUP for vector codes). */
int bifeat_produce_fit_begin(bifeat_params *p, void *stream);
int bifeat_produce_fit_end(bifeat_params *p, int64_t rows);
int bifeat_produce_quantize_check(bifeat_params *p, const uint8_t *codes, int64_t rows, int64_t row0);

/* ---- per-iteration load (Sec. 3.3).  codes: DEVICE packed table of N rows.
 * gather_codes:   out[i, :] = codes[idx[i], :]              out: DEVICE [M x row_bytes]
 * gather_dequant: out[i, j] = decode(codes[idx[i]])[j]      out: DEVICE [M x D] fp32
 * idx: DEVICE int64 [M].  M = 0 is a no-op. */
int bifeat_gather_codes(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *idx,
                        int64_t M, uint8_t *out, void *stream);
int bifeat_gather_dequant(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *idx,
                          int64_t M, float *out, void *stream);

/* bifeat_gather_dequant for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same results.  The one workspace the decode
 * kernels use (vector codes: the transposed codes of the M requested rows,
 * row_bytes * (M rounded up to 16, + 16) bytes) is a fixed array of 32 MiB
 * that is part of the library's device code, one copy per GPU, held until the
 * process ends; a request that needs more returns BIFEAT_ELIMIT (about 349 000
 * rows of 96 bytes; scalar codes use no workspace and have no limit).  The call
 * allocates nothing and never synchronises; it needs the parameters fitted or
 * set beforehand (that is when the handle's own device block is allocated) and
 * option "validate" off (BIFEAT_ENOTSUP otherwise).  Every call on a GPU, from
 * any handle or thread, shares that GPU's array: calls that overlap in time on
 * one GPU race on it - order them on one stream or with events. */
int bifeat_gather_dequant_static(bifeat_params *p, const uint8_t *codes, int64_t N,
                                 const int64_t *idx, int64_t M, float *out, void *stream);

/* ---- fused gather + decode + neighbourhood mean (Appendix A.1).
 * For v in [0, V): out[v, :] = mean over e in [indptr[v], indptr[v+1]) of
 * decode(codes[indices[e]]); the list is taken as given (repeats count with
 * multiplicity; a self-loop only if listed); an empty list gives a zero row.
 * indptr: DEVICE int64 [V+1]; indices: DEVICE int64 [E], E = indptr[V] (the host
 * passes E, which also sizes the launch); out: DEVICE [V x D] fp32.  fp32 result within 1e-5 * max(|exact|, A_j) of
 * the exact mean of the decoded values, A_j the largest decodable magnitude in
 * column j.  V = 0 is a no-op. */
int bifeat_gather_mean(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *indptr,
                       const int64_t *indices, int64_t V, int64_t E, float *out, void *stream);

/* The same with 32-bit list entries (tables of at most 2^31 - 1 rows; otherwise
 * BIFEAT_EINVAL): half the index bytes per list entry.  indices: DEVICE int32
 * [E].  Not available together with option "validate" (BIFEAT_ENOTSUP). */
int bifeat_gather_mean_i32(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *indptr,
                           const int32_t *indices, int64_t V, int64_t E, float *out, void *stream);

/* ---- the same without the division: the sum aggregator.  out[v, :] = sum over
 * the list of decode(codes[indices[e]]) (Appendix A.1 analyses the mean; the
 * sum is its unnormalised form, and with v listed among its own neighbours
 * bifeat_gather_mean is the self-loop normalisation D^-1 (A + I) written
 * there).  Arguments as bifeat_gather_mean; fp32 result within
 * 1e-5 * max(|exact|, n_v * A_j), n_v the list length. */
int bifeat_gather_sum(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *indptr,
                      const int64_t *indices, int64_t V, int64_t E, float *out, void *stream);
int bifeat_gather_sum_i32(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *indptr,
                          const int32_t *indices, int64_t V, int64_t E, float *out, void *stream);

/* ---- two rounds of the neighbourhood mean with nothing in between, straight
 * from the packed table (Appendix A.1 writes every layer's aggregation as
 * g_i = 1/|N(i)| sum_{j in N(i)} g_j and analyses how errors shrink when it is
 * applied repeatedly; this is that linear propagation for two layers of a
 * sampled minibatch).  The outer block (indptr1 [V1+1], indices1 [E1]) lists
 * table rows for each of its V1 destinations; the seed block (indptr2 [V2+1],
 * indices2 [E2], entries in [0, V1)) lists outer-block destinations for each
 * of the V2 seeds.  For v in [0, V2):
 *     out[v, :] = mean over u in list2(v) of ( mean over w in list1(u) of decode(codes[w]) ),
 * lists taken as given; an empty list1(u) is a zero row that still counts in
 * the length of list2(v); an empty list2(v) gives a zero row.  The same result
 * as bifeat_gather_mean over the outer block followed by bifeat_aggregate_rows
 * over the seed block, without the [V1 x D] fp32 rows in between ever being
 * written.  All pointers DEVICE; out: [V2 x D] fp32, within 1e-5 *
 * max(|exact|, A_j) of the exact value as for bifeat_gather_mean.
 * With option "mean_max_degree" = m (1 <= m <= 64) promising that no list of
 * either block is longer than m, scalar codes that decode affinely (uniform;
 * logarithmic of 1 or 2 bits) take a kernel that sums codes as integers and
 * keeps the running means in registers; a list that breaks the promise gives a
 * NaN row and raises the status word as described below.  Without the promise
 * that kernel takes the seeds all of whose lists have at most 64 entries and a
 * general kernel (any list length) the others.  Vector codes of power-of-two
 * width take a kernel with the codebooks in on-chip memory (any list length;
 * uses the handle's workspace like bifeat_gather_mean, sized by E1); the
 * remaining codes take the general kernel throughout.
 * Option "validate" checks both blocks first.  V2 = 0 is a no-op. */
int bifeat_gather_mean_2hop(bifeat_params *p, const uint8_t *codes, int64_t N,
                            const int64_t *indptr1, const int64_t *indices1, int64_t V1, int64_t E1,
                            const int64_t *indptr2, const int64_t *indices2, int64_t V2, int64_t E2,
                            float *out, void *stream);

/* A promise the caller made through option "mean_max_degree" and a list broke
 * (Appendix A.1's mean needs every neighbour of the list): the kernel that
 * meets such a list writes NaN into its whole output row and raises the
 * handle's status word, without any synchronisation.  The word is looked at
 * (and cleared) by the next bifeat_gather_mean / bifeat_gather_sum call on the
 * handle, which then returns BIFEAT_EINVAL without launching, and by this call:
 * BIFEAT_EINVAL if a kernel that has finished raised it since the last look,
 * else BIFEAT_OK.  wait != 0 synchronises `stream` first, so that the answer
 * covers everything enqueued on it. */
int bifeat_poll_status(bifeat_params *p, void *stream, int32_t wait);

/* Sizes the handle's workspace for gather calls of up to max_requests rows
 * (gather_dequant: M; gather_mean / gather_sum: E; gather_mean_2hop: E1), so that no later call
 * allocates.  Only vector codes use a workspace; for the other kinds this is a
 * no-op.  Not during a stream capture (BIFEAT_EHIP). */
int bifeat_reserve(bifeat_params *p, int64_t max_requests, void *stream);

/* ---- the layers after the first (Appendix A.1: every layer averages the
 * previous layer's vectors over the same neighbourhoods): the aggregation over
 * fp32 rows instead of packed codes.  For v in [0, V): out[v, :] = mean (sum != 0:
 * plain sum) over e in [indptr[v], indptr[v+1]) of x[indices[e], :], the list
 * taken as given, an empty list giving a zero row.  With the block's indices
 * local to the previous hop's output this chains after bifeat_gather_mean into
 * a multi-hop aggregation.
 * x: DEVICE [N x D] fp32 row-major; indptr: DEVICE int64 [V+1]; indices: DEVICE
 * int64 [E], each in [0, N) (the caller's contract, as for the gathers); out:
 * DEVICE [V x D] fp32, not overlapping x.  Rows are added in list order in fp32
 * with a compensated sum: within 1e-5 * max(|exact|, mean over the list of
 * |x[.., j]|) of the exact result whatever the list length (n_v times that for
 * the sum).
 * Only enqueues one kernel on `stream`.  V = 0 is a no-op. */
int bifeat_aggregate_rows(const float *x, int64_t N, int64_t D, const int64_t *indptr,
                          const int64_t *indices, int64_t V, int64_t E, int32_t sum, float *out,
                          void *stream);

/* The index contract of the calls above, checked on its own (bifeat_aggregate_rows has
 * no parameter object to carry the "validate" option): 0 <= indices[e] < N for all
 * e < E and, when indptr is not NULL, indptr[0] == 0, indptr non-decreasing,
 * indptr[V] == E.  DEVICE pointers.  Returns BIFEAT_OK or BIFEAT_EINVAL; synchronises
 * `stream` (its flag lives in a small device block taken from a per-device pool that
 * the library keeps: an allocation only when every block is in use). */
int bifeat_check_lists(const int64_t *indptr, const int64_t *indices, int64_t V, int64_t E,
                       int64_t N, void *stream);

/* ---- the aggregation scale profile (Appendix A.1 defines C^e_{i,l} and
 * C^f_{i,l}, the factors by which l rounds of averaging shrink independent
 * errors and correlated features; Appendix A.3 their ratio of means C^_L;
 * Appendix A.5 measures them by a profiling run to choose a compression
 * ratio).  The run: h_0 = x, h_l = the neighbourhood mean of h_{l-1} over the
 * whole graph (V = N, lists as given: include each node in its own list for
 * the self-loop form of Appendix A.1), and
 *     scale[l] = (1/N) sum_i ||h_l[i, :]||_2     for l = 0..layers.
 * Called with a matrix of independent unit-variance errors, scale[l]/scale[0]
 * estimates the mean of C^e_{i,l}; with unit-length feature rows it is the mean
 * of C^f_{i,l}; C^_L is the quotient of the two at l = L.
 * x, indptr, indices as above with V = N; the index contract is checked on
 * the GPU first (BIFEAT_EINVAL if broken).  work: DEVICE scratch of
 * min(layers, 2) * N * D floats, not overlapping x (may be NULL for layers = 0).
 * scale: HOST double[layers + 1].  0 <= layers <= 64.  Row lengths are
 * accumulated in fp64; h_l is stored in fp32 between rounds.  Synchronises `stream`
 * (sums and flag in a pooled device block, as for bifeat_check_lists). */
int bifeat_scale_profile(const float *x, int64_t N, int64_t D, const int64_t *indptr,
                         const int64_t *indices, int64_t E, int32_t layers, float *work,
                         double *scale, void *stream);

const char *bifeat_strerror(int status);

/* Launch tuning for measurements (no effect on results): "mean_slots" = lanes
 * that share one destination's neighbour list in bifeat_gather_mean (power of
 * two, 0 = automatic), "mean_blocks" = cap on its workgroups (0 = automatic),
 * "mean_generic" = 1 routes uniform tables through the float-accumulate
 * kernel; "mean_lean" = 0 disables the short-list kernel; "max_blocks" caps the
 * gather_dequant grid; "dequant_flat" = 1 / "vq_sliced" = 0 select the
 * unstaged decode kernels.  Two options carry information rather than tuning:
 * "mean_max_degree" = d is the caller's promise that no neighbour list of the
 * following bifeat_gather_mean calls is longer than d (0 = unknown; a sampler
 * knows its fan-out), which lets the library skip the pass that looks for
 * longer lists (a list that breaks the promise gets a row of NaNs and raises the
 * status word, see bifeat_poll_status; "validate" checks the promise up front);
 * "vq_iters" = Lloyd rounds per training chunk (1..64); "validate" = 1 checks
 * the index contract of every gather call on the GPU first (see above);
 * "row_align" = 16 (default) or 128 chooses the row stride of the packed table
 * (see the packed layout above; changes bifeat_row_bytes()).
 * Unknown names return BIFEAT_EINVAL. */
int bifeat_set_option(bifeat_params *p, const char *name, int value);

#ifdef __cplusplus
}
#endif
#endif /* BIFEAT_H */
