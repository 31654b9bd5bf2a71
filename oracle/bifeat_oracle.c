/*
 * BiFeat feature-loading path: the CPU oracle.
 *
 * TEST INFRASTRUCTURE.  A plain, slow, step-by-step implementation of what the
 * path computes, written from the paper (BiFeat, arXiv 2207.14696) to check the
 * GPU library against.  Only tests, the smoke check and the benchmark's CPU
 * baseline call it; the product never does, and the two share no code.
 *
 * What is defined by the paper, and where:
 *   - logarithmic scalar codes and their decoding     Sec. 3.1, Eq. (1), Eq. (2)
 *   - 1-bit codes (sign only, zero on the negative side)          Sec. 3.1
 *   - uniform scalar codes (evenly spaced levels), named in        Sec. 3.1
 *   - vector codes: split into parts of `width` dims, one k-means codebook of
 *     `length` entries per part, store the index      Sec. 3.2, Appendix C
 *   - per-iteration load = rows of the sampled nodes, decoded      Sec. 3.3
 *   - neighbourhood mean  g_i = (1/|N(i)|) sum_{j in N(i)} g_j     Appendix A.1
 *   - the same mean over fp32 rows (layers after the first), and the scale
 *     factors C^e, C^f, C^_L of the aggregation      Appendix A.1, A.3, A.5
 * Where the paper is silent (bit packing, the uniform scheme's exact rounding,
 * k-means initialisation) the reading taken is stated at the function.
 *
 * Precision: an integer code is decided in fp32 with individually rounded
 * operations (so a second implementation can reproduce it bit for bit);
 * decoded values and means are computed in fp64 and rounded once to fp32.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py against
 * closed forms, brute force, library routines or invariants.  Nothing in the
 * paper prints a worked numeric example, so no absolute code value is pinned
 * to a printed one.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_UNIFORM = 0, ORC_LOG = 1, ORC_VQ = 2 };

/* Everything a decoder needs.  uniform: a = min[D], b = scale[D].
 * log: a = V[2^bits] (decode table).  vq: cb = [P][len][w] codebooks. */
typedef struct {
    int32_t kind;
    int32_t bits;
    int64_t D;
    int32_t w;
    int32_t len;
    const float *a;
    const float *b;
    const float *cb;
} orc_scheme;

void orc_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int orc_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ packing
 * The paper does not fix a bit layout (Appendix C only advises against
 * elaborate packing).  Layout used: row-major; column j's `bits`-bit code sits
 * at bit offset (j*bits) mod 8 of byte floor(j*bits/8) (column 0 in the least
 * significant bits); a row occupies ceil(D*bits/8) bytes rounded up to a
 * multiple of 16, pad bytes zero.  Vector codes: byte p = index of part p. */
int64_t orc_row_bytes(int64_t ncodes, int bits) {
    int64_t nb = (ncodes * bits + 7) / 8;
    return (nb + 15) / 16 * 16;
}

void orc_pack(const uint8_t *q, int64_t rows, int64_t ncodes, int bits, uint8_t *packed) {
    int64_t rb = orc_row_bytes(ncodes, bits);
    memset(packed, 0, (size_t)(rows * rb));
    for (int64_t i = 0; i < rows; i++)
        for (int64_t j = 0; j < ncodes; j++) {
            int64_t bit = j * bits;
            packed[i * rb + bit / 8] |= (uint8_t)(q[i * ncodes + j] << (bit % 8));
        }
}

void orc_unpack(const uint8_t *packed, int64_t rows, int64_t ncodes, int bits, uint8_t *q) {
    int64_t rb = orc_row_bytes(ncodes, bits);
    unsigned mask = (1u << bits) - 1u;
    for (int64_t i = 0; i < rows; i++)
        for (int64_t j = 0; j < ncodes; j++) {
            int64_t bit = j * bits;
            q[i * ncodes + j] = (uint8_t)((packed[i * rb + bit / 8] >> (bit % 8)) & mask);
        }
}

/* Two-byte codes (vector codes with more than 256 entries per codebook;
 * Appendix C: align to whole bytes, two bytes up to 16384 entries): code j of a
 * row sits in bytes 2j (low) and 2j+1 (high); rows padded to 16 bytes as above. */
void orc_pack16(const uint16_t *q, int64_t rows, int64_t ncodes, uint8_t *packed) {
    int64_t rb = orc_row_bytes(ncodes, 16);
    memset(packed, 0, (size_t)(rows * rb));
    for (int64_t i = 0; i < rows; i++)
        for (int64_t j = 0; j < ncodes; j++) {
            packed[i * rb + 2 * j] = (uint8_t)(q[i * ncodes + j] & 0xFFu);
            packed[i * rb + 2 * j + 1] = (uint8_t)(q[i * ncodes + j] >> 8);
        }
}

void orc_unpack16(const uint8_t *packed, int64_t rows, int64_t ncodes, uint16_t *q) {
    int64_t rb = orc_row_bytes(ncodes, 16);
    for (int64_t i = 0; i < rows; i++)
        for (int64_t j = 0; j < ncodes; j++)
            q[i * ncodes + j] =
                (uint16_t)(packed[i * rb + 2 * j] | ((unsigned)packed[i * rb + 2 * j + 1] << 8));
}

/* ------------------------------------------------------- uniform scalar codes
 * Sec. 3.1 names uniform quantization (evenly spaced levels) without a
 * formula.  Reading: per column j, levels min_j + q*scale_j, q = 0..L,
 * L = 2^bits - 1, scale_j = (max_j - min_j)/L; a value maps to the nearest
 * level (ties to the even code). */

/* running per-column min/max; caller initialises mn=+inf, mx=-inf.  NaNs are
 * skipped; a zero result is stored as +0. */
void orc_fit_minmax(const float *x, int64_t rows, int64_t D, float *mn, float *mx) {
    for (int64_t i = 0; i < rows; i++)
        for (int64_t j = 0; j < D; j++) {
            float v = x[i * D + j];
            if (v < mn[j]) mn[j] = v;
            if (v > mx[j]) mx[j] = v;
        }
    for (int64_t j = 0; j < D; j++) {
        if (mn[j] == 0.0f) mn[j] = 0.0f;
        if (mx[j] == 0.0f) mx[j] = 0.0f;
    }
}

/* scale_j and its reciprocal, from fp64 arithmetic rounded once to fp32;
 * a constant column gets scale = inv = 0 (every value encodes to code 0 and
 * decodes to min exactly). */
void orc_uniform_params(const float *mn, const float *mx, int64_t D, int bits,
                        float *scale, float *inv) {
    double L = (double)((1u << bits) - 1u);
    for (int64_t j = 0; j < D; j++) {
        double range = (double)mx[j] - (double)mn[j];
        if (range > 0.0) {
            scale[j] = (float)(range / L);
            inv[j] = (float)(L / range);
        } else {
            scale[j] = 0.0f;
            inv[j] = 0.0f;
        }
    }
}

/* q = clamp(round_half_even((x - min_j) * inv_j), 0, L), each operation a
 * single fp32 rounding; NaN encodes to 0. */
void orc_uniform_encode(const float *x, int64_t rows, int64_t D, int bits,
                        const float *mn, const float *inv, uint8_t *q) {
    float L = (float)((1u << bits) - 1u);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; i++)
        for (int64_t j = 0; j < D; j++) {
            float d = x[i * D + j] - mn[j];
            float t = d * inv[j];
            float r = rintf(t);
            r = fmaxf(r, 0.0f);
            r = fminf(r, L);
            q[i * D + j] = (uint8_t)(int)r;
        }
}

/* ------------------------------------------------- logarithmic scalar codes
 * Sec. 3.1, Eq. (1): with H = 2^(k-1) and m = |x|,
 *     level l = floor( (Clip(log2 m) - e_min) / (e_max - e_min) * H ),
 *     Q(x) = H + l  on the positive side,  H - 1 - l  on the other side.
 * Readings (the equation as printed leaves these open):
 *   - l is capped at H-1 (at log2 m = e_max the printed form gives H);
 *   - side: x > 0 is positive, x <= 0 is not (the text groups zero with the
 *     negatives so that 0/1-valued features keep two distinct codes; the
 *     printed case split puts x = 0 on the positive side, which would merge
 *     0 and 1 at k = 1); NaN is treated like 0;
 *   - e_min, e_max are global (no column subscript in the paper): log2 of the
 *     smallest nonzero and of the largest finite |x|; a caller that clips a
 *     tail fraction passes a narrower pair, and Clip() clamps to it.
 * The level is decided by comparing m with the H-1 interior bin edges
 *     T_i = exp2(e_min + i*(e_max - e_min)/H), i = 1..H-1  (fp64 -> fp32),
 * l = #{i : m >= T_i}, which is Eq. (1) with the monotone log2 moved to the
 * edges; orc_log_encode_direct is the printed form, for comparison.
 * Eq. (2): Q^-1(q) = +-exp2(e_min + (l + 0.5)*(e_max - e_min)/H), minus sign on
 * the q < H side (the printed equation omits the sign; without it the two
 * halves of the code range would decode to the same values). */

/* running min of nonzero finite |x| and max of finite |x|;
 * caller initialises mmin=+inf, mmax=0 */
void orc_log_fit(const float *x, int64_t n, float *mmin, float *mmax) {
    for (int64_t i = 0; i < n; i++) {
        float m = fabsf(x[i]);
        if (!(m < INFINITY)) continue; /* inf, NaN */
        if (m > 0.0f && m < *mmin) *mmin = m;
        if (m > *mmax) *mmax = m;
    }
}

/* e_min/e_max from the fitted magnitudes; an all-zero table gets (0, 0) */
void orc_log_range(float mmin, float mmax, double *e_min, double *e_max) {
    if (!(mmax > 0.0f)) {
        *e_min = 0.0;
        *e_max = 0.0;
        return;
    }
    *e_min = log2((double)mmin);
    *e_max = log2((double)mmax);
}

/* T[H-1] bin edges and V[2^k] decode table */
void orc_log_tables(double e_min, double e_max, int k, float *T, float *V) {
    int H = 1 << (k - 1);
    double step = (e_max - e_min) / (double)H;
    for (int i = 1; i < H; i++) T[i - 1] = (float)exp2(e_min + (double)i * step);
    for (int l = 0; l < H; l++) {
        float v = (float)exp2(e_min + ((double)l + 0.5) * step);
        V[H + l] = v;
        V[H - 1 - l] = -v;
    }
}

void orc_log_encode(const float *x, int64_t n, int k, const float *T, uint8_t *q) {
    int H = 1 << (k - 1);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; i++) {
        float v = x[i];
        float m = fabsf(v);
        int l = 0;
        for (int t = 0; t < H - 1; t++)
            if (m >= T[t]) l++;
        q[i] = (uint8_t)((v > 0.0f) ? H + l : H - 1 - l);
    }
}

/* Eq. (1) as printed (log2 evaluated per element, fp64), with the readings
 * above.  Agrees with orc_log_encode except for magnitudes within rounding of
 * a bin edge. */
void orc_log_encode_direct(const float *x, int64_t n, int k, double e_min, double e_max,
                           uint8_t *q) {
    int H = 1 << (k - 1);
    for (int64_t i = 0; i < n; i++) {
        double v = (double)x[i];
        double m = fabs(v);
        int l = 0;
        if (m > 0.0 && e_max > e_min) {
            double e = log2(m);
            if (e < e_min) e = e_min;
            if (e > e_max) e = e_max;
            l = (int)floor((e - e_min) / (e_max - e_min) * (double)H);
            if (l > H - 1) l = H - 1;
        } else if (m > 0.0) {
            l = H - 1; /* e_max == e_min: every nonzero magnitude is the top edge */
        }
        q[i] = (uint8_t)((v > 0.0) ? H + l : H - 1 - l);
    }
}

/* ------------------------------------------------------------- vector codes
 * Sec. 3.2 / Appendix C: D dims are split into P = ceil(D/w) parts of w dims
 * (a short last part is zero-padded); part p of a row is replaced by the index
 * of its nearest entry in that part's codebook of `len` entries (Euclidean
 * distance; len <= 256, one byte per part as the paper advises; larger
 * codebooks and the cosine metric follow further down).
 * The squared distance is accumulated in fp32, dimension ascending, multiply
 * and add rounded separately; ties go to the lowest index. */
static int vq_nearest(const float *sub, const float *cb, int w, int len, float *best_out) {
    int best = 0;
    float bestd = INFINITY;
    for (int c = 0; c < len; c++) {
        float dist = 0.0f;
        for (int d = 0; d < w; d++) {
            float diff = sub[d] - cb[c * w + d];
            float sq = diff * diff;
            dist = dist + sq;
        }
        if (dist < bestd) {
            bestd = dist;
            best = c;
        }
    }
    if (best_out) *best_out = bestd;
    return best;
}

static void load_part(const float *row, int64_t D, int p, int w, float *sub) {
    for (int d = 0; d < w; d++) {
        int64_t j = (int64_t)p * w + d;
        sub[d] = (j < D) ? row[j] : 0.0f;
    }
}

void orc_vq_assign(const float *x, int64_t rows, int64_t D, int w, int len, const float *cb,
                   uint8_t *q) {
    int P = (int)((D + w - 1) / w);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; i++) {
        float sub[256];
        for (int p = 0; p < P; p++) {
            load_part(x + i * D, D, p, w, sub);
            q[i * P + p] = (uint8_t)vq_nearest(sub, cb + (int64_t)p * len * w, w, len, NULL);
        }
    }
}

/* Codebook training.  The paper says k-means on a uniform row sample
 * (Sec. 3.2, Appendix D) and nothing more.  Reading: per part, initial
 * entries = the first `len` pairwise distinct sub-vectors of the sample in
 * sample order (if fewer exist the rest repeat the last one and stay unused);
 * then `iters` Lloyd rounds {assign as above; entry = fp64 mean of its members
 * rounded to fp32; an entry without members keeps its value}.
 * distortion[it] = mean squared distance at round it's assignment step,
 * summed over parts (fp64). */
void orc_vq_train(const float *sample, int64_t ns, int64_t D, int w, int len, int iters,
                  float *cb, double *distortion) {
    int P = (int)((D + w - 1) / w);
    double *dpart = (double *)calloc((size_t)iters * (size_t)P, sizeof(double));
#pragma omp parallel for schedule(dynamic)
    for (int p = 0; p < P; p++) {
        float *C = cb + (int64_t)p * len * w;
        float sub[256];
        int have = 0;
        for (int64_t i = 0; i < ns && have < len; i++) {
            load_part(sample + i * D, D, p, w, sub);
            int dup = 0;
            for (int c = 0; c < have && !dup; c++)
                dup = (memcmp(C + c * w, sub, sizeof(float) * (size_t)w) == 0);
            if (!dup) memcpy(C + (have++) * w, sub, sizeof(float) * (size_t)w);
        }
        for (int c = have; c < len; c++)
            memcpy(C + c * w, C + (have - 1) * w, sizeof(float) * (size_t)w);

        double *sum = (double *)malloc(sizeof(double) * (size_t)len * (size_t)w);
        int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)len);
        for (int it = 0; it < iters; it++) {
            memset(sum, 0, sizeof(double) * (size_t)len * (size_t)w);
            memset(cnt, 0, sizeof(int64_t) * (size_t)len);
            double dsum = 0.0;
            for (int64_t i = 0; i < ns; i++) {
                float bd;
                load_part(sample + i * D, D, p, w, sub);
                int c = vq_nearest(sub, C, w, len, &bd);
                dsum += (double)bd;
                cnt[c]++;
                for (int d = 0; d < w; d++) sum[c * w + d] += (double)sub[d];
            }
            for (int c = 0; c < len; c++)
                if (cnt[c] > 0)
                    for (int d = 0; d < w; d++)
                        C[c * w + d] = (float)(sum[c * w + d] / (double)cnt[c]);
            dpart[(size_t)it * (size_t)P + (size_t)p] = dsum / (double)ns;
        }
        free(sum);
        free(cnt);
    }
    for (int it = 0; it < iters; it++) {
        distortion[it] = 0.0;
        for (int p = 0; p < P; p++) distortion[it] += dpart[(size_t)it * (size_t)P + (size_t)p];
    }
    free(dpart);
}

/* ---- the variants of Sec. 3.2 / Appendix C beyond one-byte Euclidean codes
 * Metric.  Sec. 3.2 allows Euclidean distance or cosine similarity for the
 * nearest-entry search and says no more.  Reading for cosine: the part takes
 * the entry with the largest (x . C_c) / |C_c|; the row's own norm is a common
 * positive factor and is left out (an all-zero part scores 0 everywhere and
 * takes entry 0); an all-zero entry scores 0.  The dot product is accumulated
 * in fp32, dimension ascending, multiply and add rounded separately, then
 * multiplied by rnorm_c = fp32(1 / sqrt(sum_d C_cd^2)) with the sum and the
 * root in fp64; ties go to the lowest index.  Codebook entries stay plain
 * arithmetic means of their members and decoding returns the entry as it is.
 * Codebook size.  More than 256 entries (up to 16384) take two bytes per part. */
enum { ORC_L2 = 0, ORC_COSINE = 1 };

void orc_vq_rnorm(const float *cb, int64_t entries, int w, float *rnorm) {
    for (int64_t c = 0; c < entries; c++) {
        double ss = 0.0;
        for (int d = 0; d < w; d++) ss += (double)cb[c * w + d] * (double)cb[c * w + d];
        rnorm[c] = (ss > 0.0) ? (float)(1.0 / sqrt(ss)) : 0.0f;
    }
}

static int vq_most_similar(const float *sub, const float *cb, const float *rnorm, int w, int len) {
    int best = 0;
    float bests = -INFINITY;
    for (int c = 0; c < len; c++) {
        float dot = 0.0f;
        for (int d = 0; d < w; d++) {
            float pr = sub[d] * cb[c * w + d];
            dot = dot + pr;
        }
        float score = dot * rnorm[c];
        if (score > bests) {
            bests = score;
            best = c;
        }
    }
    return best;
}

/* codes as 16-bit integers whatever the codebook size; metric: ORC_L2 / ORC_COSINE */
void orc_vq_assign16(const float *x, int64_t rows, int64_t D, int w, int len, const float *cb,
                     int metric, uint16_t *q) {
    int P = (int)((D + w - 1) / w);
    float *rnorm = NULL;
    if (metric == ORC_COSINE) {
        rnorm = (float *)malloc(sizeof(float) * (size_t)P * (size_t)len);
        orc_vq_rnorm(cb, (int64_t)P * len, w, rnorm);
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; i++) {
        float sub[256];
        for (int p = 0; p < P; p++) {
            const float *C = cb + (int64_t)p * len * w;
            load_part(x + i * D, D, p, w, sub);
            q[i * P + p] = (uint16_t)(metric == ORC_COSINE
                                          ? vq_most_similar(sub, C, rnorm + (int64_t)p * len, w, len)
                                          : vq_nearest(sub, C, w, len, NULL));
        }
    }
    free(rnorm);
}

/* Lloyd rounds as orc_vq_train, the assignment step by `metric`.  distortion[it]
 * is the mean squared Euclidean distance between a part and its assigned entry
 * (the decoding error), fp64, summed over parts, for either metric. */
void orc_vq_train_metric(const float *sample, int64_t ns, int64_t D, int w, int len, int iters,
                         int metric, float *cb, double *distortion) {
    int P = (int)((D + w - 1) / w);
    double *dpart = (double *)calloc((size_t)iters * (size_t)P, sizeof(double));
#pragma omp parallel for schedule(dynamic)
    for (int p = 0; p < P; p++) {
        float *C = cb + (int64_t)p * len * w;
        float sub[256];
        int have = 0;
        for (int64_t i = 0; i < ns && have < len; i++) {
            load_part(sample + i * D, D, p, w, sub);
            int dup = 0;
            for (int c = 0; c < have && !dup; c++)
                dup = (memcmp(C + c * w, sub, sizeof(float) * (size_t)w) == 0);
            if (!dup) memcpy(C + (have++) * w, sub, sizeof(float) * (size_t)w);
        }
        for (int c = have; c < len; c++)
            memcpy(C + c * w, C + (have - 1) * w, sizeof(float) * (size_t)w);

        double *sum = (double *)malloc(sizeof(double) * (size_t)len * (size_t)w);
        int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)len);
        float *rnorm = (float *)malloc(sizeof(float) * (size_t)len);
        for (int it = 0; it < iters; it++) {
            memset(sum, 0, sizeof(double) * (size_t)len * (size_t)w);
            memset(cnt, 0, sizeof(int64_t) * (size_t)len);
            if (metric == ORC_COSINE) orc_vq_rnorm(C, len, w, rnorm);
            double dsum = 0.0;
            for (int64_t i = 0; i < ns; i++) {
                load_part(sample + i * D, D, p, w, sub);
                int c = (metric == ORC_COSINE) ? vq_most_similar(sub, C, rnorm, w, len)
                                               : vq_nearest(sub, C, w, len, NULL);
                for (int d = 0; d < w; d++) {
                    double diff = (double)sub[d] - (double)C[c * w + d];
                    dsum += diff * diff;
                }
                cnt[c]++;
                for (int d = 0; d < w; d++) sum[c * w + d] += (double)sub[d];
            }
            for (int c = 0; c < len; c++)
                if (cnt[c] > 0)
                    for (int d = 0; d < w; d++)
                        C[c * w + d] = (float)(sum[c * w + d] / (double)cnt[c]);
            dpart[(size_t)it * (size_t)P + (size_t)p] = dsum / (double)ns;
        }
        free(sum);
        free(cnt);
        free(rnorm);
    }
    for (int it = 0; it < iters; it++) {
        distortion[it] = 0.0;
        for (int p = 0; p < P; p++) distortion[it] += dpart[(size_t)it * (size_t)P + (size_t)p];
    }
    free(dpart);
}

/* ------------------------------------------------------------------ decoding */
static inline unsigned code_at(const uint8_t *row, int64_t j, int bits) {
    int64_t bit = j * bits;
    return (row[bit / 8] >> (bit % 8)) & ((1u << bits) - 1u);
}

/* one packed row -> D decoded values (fp64) */
static void decode_row(const orc_scheme *s, const uint8_t *row, double *out) {
    if (s->kind == ORC_UNIFORM) {
        for (int64_t j = 0; j < s->D; j++)
            out[j] = (double)s->a[j] + (double)code_at(row, j, s->bits) * (double)s->b[j];
    } else if (s->kind == ORC_LOG) {
        for (int64_t j = 0; j < s->D; j++) out[j] = (double)s->a[code_at(row, j, s->bits)];
    } else {
        for (int64_t j = 0; j < s->D; j++) {
            int64_t p = j / s->w, d = j % s->w;
            int64_t q = (s->len > 256) ? (int64_t)(row[2 * p] | ((unsigned)row[2 * p + 1] << 8))
                                       : (int64_t)row[p];
            out[j] = (double)s->cb[(p * s->len + q) * s->w + d];
        }
    }
}

int64_t orc_scheme_row_bytes(const orc_scheme *s) {
    if (s->kind == ORC_VQ) return orc_row_bytes((s->D + s->w - 1) / s->w, s->len > 256 ? 16 : 8);
    return orc_row_bytes(s->D, s->bits);
}

/* ---------------------------------------------------- the per-iteration load
 * Sec. 3.3: fetch the compressed rows of the sampled nodes, decode them.    */
void orc_gather_codes(const uint8_t *codes, int64_t rb, const int64_t *idx, int64_t M,
                      uint8_t *out) {
    for (int64_t i = 0; i < M; i++) memcpy(out + i * rb, codes + idx[i] * rb, (size_t)rb);
}

void orc_gather_dequant(const orc_scheme *s, const uint8_t *codes, const int64_t *idx, int64_t M,
                        float *out) {
    int64_t rb = orc_scheme_row_bytes(s), D = s->D;
#pragma omp parallel
    {
        double *tmp = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(static)
        for (int64_t i = 0; i < M; i++) {
            decode_row(s, codes + idx[i] * rb, tmp);
            for (int64_t j = 0; j < D; j++) out[i * D + j] = (float)tmp[j];
        }
        free(tmp);
    }
}

/* The unnormalised form of the aggregation below (the sum aggregator of
 * GraphSAGE-style layers; Appendix A.1 analyses the mean): out[v] = sum over the
 * listed neighbours of their decoded rows, in list order, fp64, one rounding to
 * fp32; an empty list gives a zero row. */
void orc_gather_sum(const orc_scheme *s, const uint8_t *codes, const int64_t *indptr,
                    const int64_t *indices, int64_t V, float *out) {
    int64_t rb = orc_scheme_row_bytes(s), D = s->D;
#pragma omp parallel
    {
        double *tmp = (double *)malloc(sizeof(double) * (size_t)D);
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 64)
        for (int64_t v = 0; v < V; v++) {
            for (int64_t j = 0; j < D; j++) acc[j] = 0.0;
            for (int64_t e = indptr[v]; e < indptr[v + 1]; e++) {
                decode_row(s, codes + indices[e] * rb, tmp);
                for (int64_t j = 0; j < D; j++) acc[j] += tmp[j];
            }
            for (int64_t j = 0; j < D; j++) out[v * D + j] = (float)acc[j];
        }
        free(tmp);
        free(acc);
    }
}

/* Appendix A.1: out[v] = (1/|N(v)|) * sum over the listed neighbours of their
 * decoded rows, in list order, fp64, one rounding to fp32.  The list is taken
 * as given (repeats count with multiplicity; a self-loop is present only if
 * the caller lists it); an empty list gives a zero row. */
void orc_gather_mean(const orc_scheme *s, const uint8_t *codes, const int64_t *indptr,
                     const int64_t *indices, int64_t V, float *out) {
    int64_t rb = orc_scheme_row_bytes(s), D = s->D;
#pragma omp parallel
    {
        double *tmp = (double *)malloc(sizeof(double) * (size_t)D);
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 64)
        for (int64_t v = 0; v < V; v++) {
            int64_t n = indptr[v + 1] - indptr[v];
            for (int64_t j = 0; j < D; j++) acc[j] = 0.0;
            for (int64_t e = indptr[v]; e < indptr[v + 1]; e++) {
                decode_row(s, codes + indices[e] * rb, tmp);
                for (int64_t j = 0; j < D; j++) acc[j] += tmp[j];
            }
            for (int64_t j = 0; j < D; j++)
                out[v * D + j] = (n > 0) ? (float)(acc[j] / (double)n) : 0.0f;
        }
        free(tmp);
        free(acc);
    }
}

/* ------------------------------- later layers and the aggregation scale factors
 * Appendix A.1: every layer after the first aggregates the previous layer's
 * rows in the same way, g_i = (1/|N(i)|) sum_{j in N(i)} g_j, over fp32 rows
 * instead of packed codes.  out[v] = mean (sum != 0: plain sum) of the listed
 * rows of x, in list order, fp64, one rounding to fp32; an empty list gives a
 * zero row; repeats count with multiplicity. */
void orc_aggregate_rows(const float *x, int64_t D, const int64_t *indptr, const int64_t *indices,
                        int64_t V, int sum, float *out) {
#pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 64)
        for (int64_t v = 0; v < V; v++) {
            int64_t n = indptr[v + 1] - indptr[v];
            for (int64_t j = 0; j < D; j++) acc[j] = 0.0;
            for (int64_t e = indptr[v]; e < indptr[v + 1]; e++) {
                const float *row = x + indices[e] * D;
                for (int64_t j = 0; j < D; j++) acc[j] += (double)row[j];
            }
            for (int64_t j = 0; j < D; j++) {
                double r = sum ? acc[j] : (n > 0 ? acc[j] / (double)n : 0.0);
                out[v * D + j] = (float)r;
            }
        }
        free(acc);
    }
}

/* Two rounds of Appendix A.1's averaging with nothing in between, straight from
 * the packed table: g1[u] = (1/|N1(u)|) sum_{w in N1(u)} decode(codes[w]) for the
 * destinations u of the outer block (lists of table rows), and
 * out[v] = (1/|N2(v)|) sum_{u in N2(v)} g1[u] for the destinations v of the seed
 * block (lists of outer-block destinations, 0 <= u < V1).  Lists in the order
 * given, repeats with multiplicity; an empty N1(u) makes g1[u] a zero row that
 * still counts in |N2(v)|; an empty N2(v) gives a zero row.  fp64 throughout,
 * g1 is not rounded, one rounding to fp32 at the end. */
void orc_gather_mean_2hop(const orc_scheme *s, const uint8_t *codes, const int64_t *indptr1,
                          const int64_t *indices1, const int64_t *indptr2, const int64_t *indices2,
                          int64_t V2, float *out) {
    int64_t rb = orc_scheme_row_bytes(s), D = s->D;
#pragma omp parallel
    {
        double *tmp = (double *)malloc(sizeof(double) * (size_t)D);
        double *g1 = (double *)malloc(sizeof(double) * (size_t)D);
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 16)
        for (int64_t v = 0; v < V2; v++) {
            int64_t n2 = indptr2[v + 1] - indptr2[v];
            for (int64_t j = 0; j < D; j++) acc[j] = 0.0;
            for (int64_t e2 = indptr2[v]; e2 < indptr2[v + 1]; e2++) {
                int64_t u = indices2[e2];
                int64_t n1 = indptr1[u + 1] - indptr1[u];
                for (int64_t j = 0; j < D; j++) g1[j] = 0.0;
                for (int64_t e1 = indptr1[u]; e1 < indptr1[u + 1]; e1++) {
                    decode_row(s, codes + indices1[e1] * rb, tmp);
                    for (int64_t j = 0; j < D; j++) g1[j] += tmp[j];
                }
                if (n1 > 0)
                    for (int64_t j = 0; j < D; j++) acc[j] += g1[j] / (double)n1;
            }
            for (int64_t j = 0; j < D; j++)
                out[v * D + j] = (n2 > 0) ? (float)(acc[j] / (double)n2) : 0.0f;
        }
        free(tmp);
        free(g1);
        free(acc);
    }
}

/* Appendix A.1 defines, per node i and depth l, the factors C^e_{i,l} and
 * C^f_{i,l}: by how much l rounds of neighbourhood averaging shrink a
 * quantisation error (independent between nodes) and the features themselves
 * (correlated between neighbours); the appendix's analysis of depth and graph
 * structure reports their means over the nodes and the ratio
 * C^_L = mean_i C^e_{i,L} / mean_i C^f_{i,L}, and says they are obtained by a
 * profiling run rather than from graph statistics.  That run, as read here:
 * push a matrix through `layers` rounds of the averaging alone (no weights, no
 * activation: the factors are defined as the effect of the aggregation) over
 * the whole graph, lists taken as given (Appendix A.1 uses lists that include
 * the node itself), and record how long the rows still are:
 *     h_0 = x,  h_l[i] = (1/|N(i)|) sum_{j in N(i)} h_{l-1}[j]  (empty list: 0),
 *     scale[l] = (1/n) sum_i ||h_l[i]||_2 ,  l = 0..layers.
 * With x = an error matrix of independent unit-variance entries,
 * scale[l]/scale[0] estimates mean_i C^e_{i,l}; with x = the unit-length
 * feature rows it is mean_i C^f_{i,l}.  Everything in fp64, nothing rounded
 * between the rounds. */
void orc_scale_profile(const float *x, int64_t n, int64_t D, const int64_t *indptr,
                       const int64_t *indices, int layers, double *scale) {
    size_t total = (size_t)n * (size_t)D;
    double *h = (double *)malloc(sizeof(double) * (total ? total : 1));
    double *g = (double *)malloc(sizeof(double) * (total ? total : 1));
    for (size_t t = 0; t < total; t++) h[t] = (double)x[t];
    for (int l = 0; l <= layers; l++) {
        if (l > 0) {
#pragma omp parallel for schedule(dynamic, 64)
            for (int64_t i = 0; i < n; i++) {
                int64_t cnt = indptr[i + 1] - indptr[i];
                for (int64_t j = 0; j < D; j++) g[i * D + j] = 0.0;
                for (int64_t e = indptr[i]; e < indptr[i + 1]; e++)
                    for (int64_t j = 0; j < D; j++) g[i * D + j] += h[indices[e] * D + j];
                if (cnt > 0)
                    for (int64_t j = 0; j < D; j++) g[i * D + j] /= (double)cnt;
            }
            double *t = h; h = g; g = t;
        }
        double s = 0.0;
        for (int64_t i = 0; i < n; i++) {
            double q = 0.0;
            for (int64_t j = 0; j < D; j++) q += h[i * D + j] * h[i * D + j];
            s += sqrt(q);
        }
        scale[l] = n > 0 ? s / (double)n : 0.0;
    }
    free(h);
    free(g);
}
