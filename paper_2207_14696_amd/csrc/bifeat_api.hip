// C ABI of the library: argument checks, the quantizer-parameter object, and
// dispatch to the kernels.  Everything that touches data runs in the kernels of
// fit_quantize.hip / gather.hip / gather_mean.hip; this file only marshals.
#include <math.h>
#include <string.h>

#include <map>
#include <mutex>
#include <new>
#include <string>

#include "common.hpp"

namespace {

thread_local std::string g_hip_error;

int hip_fail(hipError_t e, const char *what) {
    g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return BIFEAT_EHIP;
}

#define BF_HIP(call)                                  \
    do {                                              \
        hipError_t e_ = (call);                       \
        if (e_ != hipSuccess) return hip_fail(e_, #call); \
    } while (0)

bool scheme_ok(const bifeat_scheme *s, int64_t D) {
    if (!s || D <= 0 || D > (int64_t)1 << 24) return false;
    if (s->kind == BIFEAT_SQ_UNIFORM || s->kind == BIFEAT_SQ_LOG)
        return s->bits == 1 || s->bits == 2 || s->bits == 4 || s->bits == 8;
    if (s->kind == BIFEAT_VQ)
        return s->vq_width >= 1 && s->vq_width <= 128 && s->vq_length >= 2 &&
               s->vq_length <= 16384 &&
               (s->vq_metric == BIFEAT_VQ_L2 || s->vq_metric == BIFEAT_VQ_COSINE);
    return false;
}

int64_t round16(int64_t n) { return (n + 15) / 16 * 16; }

// Row stride for the table's alignment option.  16: rows back to back.  128: rows of up to 128
// bytes take the next power of two (a row then never straddles a 128-byte line), longer rows a
// whole number of lines.
int64_t row_stride(int64_t payload, int align) {
    if (align < 128) return payload;
    if (payload <= 128) {
        int64_t s = 16;
        while (s < payload) s *= 2;
        return s;
    }
    return (payload + 127) / 128 * 128;
}

// allocate the device block on first GPU use
int ensure_device(bifeat_params *p) {
    if (p->d_block) return BIFEAT_OK;
    BF_HIP(hipGetDevice(&p->device));
    const int64_t D = p->D;
    size_t nfloat = 0, nfit = 0;
    if (p->scheme.kind == BIFEAT_SQ_UNIFORM) { nfloat = 4 * D; nfit = 2 * D; }
    else if (p->scheme.kind == BIFEAT_SQ_LOG) {
        // bin edges, decode table and, for 1-bit codes, the table again as a per-column
        // affine map (decode = V[0] + q*(V[1]-V[0])) for the integer-sum mean kernels
        nfloat = 128 + 256 + (p->scheme.bits == 1 ? 2 * D : p->scheme.bits == 2 ? 4 * D : 0);
        nfit = 4 + 2 * 2 * bf::kLogHistBins;
    }
    else nfloat = (size_t)p->P * p->scheme.vq_length * (2 * p->scheme.vq_width + 2) + 64;
    nfloat = (nfloat + 3) / 4 * 4;
    nfit = (nfit + 3) / 4 * 4;
    void *blk = nullptr;
    const size_t bytes = sizeof(float) * nfloat + sizeof(int32_t) * nfit + 128;  // zero row + check flag
    BF_HIP(hipMalloc(&blk, bytes));
    BF_HIP(hipMemset(blk, 0, bytes));
    p->d_block = (float *)blk;
    if (p->scheme.kind == BIFEAT_SQ_UNIFORM) {
        p->d_min = p->d_block;
        p->d_scale = p->d_min + D;
        p->d_inv = p->d_scale + D;
        p->d_max = p->d_inv + D;
    } else if (p->scheme.kind == BIFEAT_SQ_LOG) {
        p->d_T = p->d_block;
        p->d_V = p->d_block + 128;
        if (p->scheme.bits == 1) {
            p->d_min = p->d_V + 256;
            p->d_scale = p->d_min + D;
        } else if (p->scheme.bits == 2) {  // per bit column: 2*D entries each
            p->d_min = p->d_V + 256;
            p->d_scale = p->d_min + 2 * D;
        }
    } else {
        const size_t ncb = (size_t)p->P * p->scheme.vq_length * p->scheme.vq_width;
        const size_t nent = (size_t)p->P * p->scheme.vq_length;
        p->d_cb = p->d_block;
        p->d_rnorm = p->d_block + ncb;
        p->d_train = p->d_rnorm + nent;
        p->d_dist = p->d_train + ncb + nent;
    }
    p->d_fit = reinterpret_cast<int32_t *>(p->d_block + nfloat);
    if (p->scheme.kind == BIFEAT_SQ_LOG) p->d_hist = reinterpret_cast<unsigned long long *>(p->d_fit + 4);
    p->d_zero = reinterpret_cast<uint8_t *>(p->d_fit + nfit);
    // the status word: pinned host memory that the kernels write through its device mapping
    void *hs = nullptr, *ds = nullptr;
    BF_HIP(hipHostMalloc(&hs, 64, hipHostMallocMapped));
    memset(hs, 0, 64);
    BF_HIP(hipHostGetDevicePointer(&ds, hs, 0));
    p->h_status = (int32_t *)hs;
    p->d_status = (int32_t *)ds;
    return BIFEAT_OK;
}

// Small zeroed device blocks for the calls that have no handle to keep one in
// (bifeat_check_lists, bifeat_scale_profile): taken from a per-device pool and given back,
// so that a call allocates only when every block of its device is in use.
constexpr size_t kPoolBlockBytes = 1024;
std::mutex g_pool_mutex;
std::map<int, std::vector<void *>> g_pool;

int pool_take(void **out) {
    int dev = 0;
    BF_HIP(hipGetDevice(&dev));
    {
        std::lock_guard<std::mutex> lock(g_pool_mutex);
        std::vector<void *> &free_blocks = g_pool[dev];
        if (!free_blocks.empty()) {
            *out = free_blocks.back();
            free_blocks.pop_back();
            return BIFEAT_OK;
        }
    }
    BF_HIP(hipMalloc(out, kPoolBlockBytes));
    return BIFEAT_OK;
}

void pool_give(void *blk) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return;
    std::lock_guard<std::mutex> lock(g_pool_mutex);
    g_pool[dev].push_back(blk);
}

// the status word raised by a kernel of an earlier call on this handle, cleared
int take_status(bifeat_params *p) {
    if (!p->h_status) return 0;
    return __atomic_exchange_n(p->h_status, 0, __ATOMIC_ACQ_REL);
}

// log scheme: bin edges and decode table from (e_min, e_max), fp64 -> fp32
void build_log_tables(bifeat_params *p) {
    const int k = p->scheme.bits, H = 1 << (k - 1);
    const double step = (p->e_max - p->e_min) / (double)H;
    p->h_T.assign((size_t)(H > 1 ? H - 1 : 0), 0.f);
    p->h_V.assign((size_t)1 << k, 0.f);
    for (int i = 1; i < H; i++) p->h_T[i - 1] = (float)exp2(p->e_min + (double)i * step);
    for (int l = 0; l < H; l++) {
        float v = (float)exp2(p->e_min + ((double)l + 0.5) * step);
        p->h_V[H + l] = v;
        p->h_V[H - 1 - l] = -v;
    }
}

int upload_log(bifeat_params *p) {
    int rc = ensure_device(p);
    if (rc) return rc;
    if (!p->h_T.empty())
        BF_HIP(hipMemcpy(p->d_T, p->h_T.data(), sizeof(float) * p->h_T.size(), hipMemcpyHostToDevice));
    BF_HIP(hipMemcpy(p->d_V, p->h_V.data(), sizeof(float) * p->h_V.size(), hipMemcpyHostToDevice));
    if (p->scheme.bits == 1) {
        // V[1] = -V[0]: the difference and V[0] + 1*(V[1]-V[0]) are exact
        std::vector<float> col((size_t)2 * p->D);
        for (int64_t j = 0; j < p->D; j++) {
            col[j] = p->h_V[0];
            col[p->D + j] = p->h_V[1] - p->h_V[0];
        }
        BF_HIP(hipMemcpy(p->d_min, col.data(), sizeof(float) * col.size(), hipMemcpyHostToDevice));
    } else if (p->scheme.bits == 2) {
        // decoded sum = (v1 - v0)*S0 - n*v1 + (v0 + v1)*S1 over the two bit planes of a column
        // (V = [-v1, -v0, v0, v1]): bit column 2t maps S0, bit column 2t+1 maps S1
        const double v0 = p->h_V[2], v1 = p->h_V[3];
        std::vector<float> col((size_t)4 * p->D);
        for (int64_t j = 0; j < p->D; j++) {
            col[2 * j] = (float)-v1;
            col[2 * j + 1] = 0.0f;
            col[2 * p->D + 2 * j] = (float)(v1 - v0);
            col[2 * p->D + 2 * j + 1] = (float)(v0 + v1);
        }
        BF_HIP(hipMemcpy(p->d_min, col.data(), sizeof(float) * col.size(), hipMemcpyHostToDevice));
    }
    return BIFEAT_OK;
}

// uniform scheme: bring the device-side fit results to the host copies
int sync_uniform_host(bifeat_params *p) {
    if (p->host_valid) return BIFEAT_OK;
    const size_t D = (size_t)p->D;
    p->h_min.resize(D); p->h_max.resize(D); p->h_scale.resize(D); p->h_inv.resize(D);
    BF_HIP(hipDeviceSynchronize());
    BF_HIP(hipMemcpy(p->h_min.data(), p->d_min, 4 * D, hipMemcpyDeviceToHost));
    BF_HIP(hipMemcpy(p->h_max.data(), p->d_max, 4 * D, hipMemcpyDeviceToHost));
    BF_HIP(hipMemcpy(p->h_scale.data(), p->d_scale, 4 * D, hipMemcpyDeviceToHost));
    BF_HIP(hipMemcpy(p->h_inv.data(), p->d_inv, 4 * D, hipMemcpyDeviceToHost));
    p->host_valid = true;
    return BIFEAT_OK;
}

// cosine metric: reciprocal entry norms from the host copy of the codebooks,
// fp32(1/sqrt(sum of squares)) with the sum and the root in fp64
int upload_rnorm(bifeat_params *p) {
    if (p->scheme.vq_metric != BIFEAT_VQ_COSINE) return BIFEAT_OK;
    const size_t nent = (size_t)p->P * p->scheme.vq_length, w = (size_t)p->scheme.vq_width;
    p->h_rnorm.resize(nent);
    for (size_t c = 0; c < nent; c++) {
        double ss = 0.0;
        for (size_t d = 0; d < w; d++) ss += (double)p->h_cb[c * w + d] * (double)p->h_cb[c * w + d];
        p->h_rnorm[c] = ss > 0.0 ? (float)(1.0 / sqrt(ss)) : 0.0f;
    }
    BF_HIP(hipMemcpy(p->d_rnorm, p->h_rnorm.data(), 4 * nent, hipMemcpyHostToDevice));
    return BIFEAT_OK;
}

int sync_codebooks_host(bifeat_params *p) {
    if (p->host_valid) return BIFEAT_OK;
    const size_t n = (size_t)p->P * p->scheme.vq_length * p->scheme.vq_width;
    p->h_cb.resize(n);
    BF_HIP(hipDeviceSynchronize());
    BF_HIP(hipMemcpy(p->h_cb.data(), p->d_cb, 4 * n, hipMemcpyDeviceToHost));
    p->host_valid = true;
    return BIFEAT_OK;
}

// first bin whose cumulative count exceeds `rank`; `before` = count below that bin
bool walk_histogram(const unsigned long long *h, int bins, unsigned long long rank, uint32_t *bin,
                    unsigned long long *before) {
    unsigned long long cum = 0;
    for (int b = 0; b < bins; b++) {
        if (rank < cum + h[b]) {
            *bin = (uint32_t)b;
            *before = cum;
            return true;
        }
        cum += h[b];
    }
    return false;
}

int finish_log(bifeat_params *p) {
    build_log_tables(p);
    int rc = upload_log(p);
    if (rc) return rc;
    p->host_valid = true;
    p->fit_open = false;
    p->fitted = true;
    return BIFEAT_OK;
}

// one step of the three-pass radix selection (digits of 11, 11 and 9 bits)
int finalize_log_clipped(bifeat_params *p, hipStream_t s) {
    std::vector<unsigned long long> h((size_t)2 * bf::kLogHistBins);
    BF_HIP(hipMemcpyAsync(h.data(), p->d_hist, sizeof(unsigned long long) * h.size(),
                          hipMemcpyDeviceToHost, s));
    BF_HIP(hipStreamSynchronize(s));
    const unsigned long long *h0 = h.data(), *h1 = h.data() + bf::kLogHistBins;
    unsigned long long before = 0;
    uint32_t bin = 0;
    if (p->fit_pass == 0) {
        unsigned long long n = 0;
        for (int b = 0; b < bf::kLogHistBins; b++) n += h0[b];
        if (n == 0) {  // nothing but zeros / non-finite values
            p->e_min = p->e_max = 0.0;
            return finish_log(p);
        }
        const double f = p->clip_fraction;
        p->clip_rank[0] = (unsigned long long)floor(f * (double)(n - 1));
        p->clip_rank[1] = (unsigned long long)ceil((1.0 - f) * (double)(n - 1));
        for (int t = 0; t < 2; t++) {
            if (!walk_histogram(h0, bf::kLogHistBins, p->clip_rank[t], &bin, &before)) return BIFEAT_EINVAL;
            p->clip_prefix[t] = bin;
            p->clip_rank[t] -= before;
        }
    } else {
        const int bins = p->fit_pass == 1 ? bf::kLogHistBins : 512, shift = p->fit_pass == 1 ? 11 : 9;
        for (int t = 0; t < 2; t++) {
            if (!walk_histogram(t ? h1 : h0, bins, p->clip_rank[t], &bin, &before)) {
                p->fit_open = false;  // the passes did not see the same data
                return BIFEAT_EINVAL;
            }
            p->clip_prefix[t] = (p->clip_prefix[t] << shift) | bin;
            p->clip_rank[t] -= before;
        }
        if (p->fit_pass == 2) {
            float lo, hi;
            memcpy(&lo, &p->clip_prefix[0], 4);
            memcpy(&hi, &p->clip_prefix[1], 4);
            p->e_min = log2((double)lo);
            p->e_max = log2((double)hi);
            return finish_log(p);
        }
    }
    p->fit_pass++;
    bf::launch_log_hist_reset(p, s);
    return BIFEAT_FIT_AGAIN;
}

bool dtype_ok(int32_t d) { return d == BIFEAT_F32 || d == BIFEAT_F16; }

}  // namespace

extern "C" {

int bifeat_params_create(const bifeat_scheme *scheme, int64_t D, bifeat_params **out) {
    if (!out) return BIFEAT_EINVAL;
    *out = nullptr;
    if (!scheme_ok(scheme, D)) return BIFEAT_EINVAL;
    bifeat_params *p = new (std::nothrow) bifeat_params();
    if (!p) return BIFEAT_EINVAL;
    p->scheme = *scheme;
    p->D = D;
    if (scheme->kind == BIFEAT_VQ) {
        p->P = (int)((D + scheme->vq_width - 1) / scheme->vq_width);
        p->ncodes = p->P;
        p->cbytes = scheme->vq_length <= 256 ? 1 : 2;
        p->payload = round16((int64_t)p->P * p->cbytes);
        p->scheme.bits = 8 * p->cbytes;
    } else {
        p->ncodes = D;
        p->payload = round16((D * scheme->bits + 7) / 8);
    }
    p->rb = row_stride(p->payload, p->opt_row_align);
    *out = p;
    return BIFEAT_OK;
}

void bifeat_params_destroy(bifeat_params *p) {
    if (!p) return;
    if (p->d_block) (void)hipFree(p->d_block);
    if (p->d_scratch) (void)hipFree(p->d_scratch);
    for (void *q : p->retired) (void)hipFree(q);
    if (p->h_status) (void)hipHostFree(p->h_status);
    delete p;
}

int64_t bifeat_row_bytes(const bifeat_params *p) { return p ? p->rb : BIFEAT_EINVAL; }
int64_t bifeat_codes_per_row(const bifeat_params *p) { return p ? p->ncodes : BIFEAT_EINVAL; }

int bifeat_set_option(bifeat_params *p, const char *name, int value) {
    if (!p || !name || value < 0) return BIFEAT_EINVAL;
    if (!strcmp(name, "mean_slots")) p->opt_mean_slots = value;
    else if (!strcmp(name, "mean_blocks")) p->opt_mean_blocks = value;
    else if (!strcmp(name, "mean_generic")) p->opt_mean_generic = value;
    else if (!strcmp(name, "validate")) p->opt_validate = value;
    else if (!strcmp(name, "max_blocks")) p->opt_max_blocks = value;
    else if (!strcmp(name, "dequant_flat")) p->opt_dequant_flat = value;
    else if (!strcmp(name, "mean_lean")) p->opt_mean_lean = value;
    else if (!strcmp(name, "vq_sliced")) p->opt_vq_sliced = value;
    else if (!strcmp(name, "vq_iters") && value >= 1 && value <= 64) p->opt_vq_iters = value;
    else if (!strcmp(name, "mean_max_degree")) p->opt_mean_max_degree = value;
    else if (!strcmp(name, "row_align") && (value == 16 || value == 128)) {
        p->opt_row_align = value;
        p->rb = row_stride(p->payload, value);
    }
    else return BIFEAT_EINVAL;
    return BIFEAT_OK;
}

int bifeat_fit_reset(bifeat_params *p, void *stream) {
    if (!p) return BIFEAT_EINVAL;
    int rc = ensure_device(p);
    if (rc) return rc;
    if (p->scheme.kind == BIFEAT_VQ) p->vq_seeded = false;
    else BF_HIP(bf::launch_fit_reset(p, (hipStream_t)stream));
    if (p->scheme.kind == BIFEAT_SQ_LOG && p->clip_fraction > 0.0) {
        p->fit_pass = 0;
        p->clip_prefix[0] = p->clip_prefix[1] = 0;
        bf::launch_log_hist_reset(p, (hipStream_t)stream);
    }
    p->fit_open = true;
    p->fit_rows = 0;
    p->fitted = false;
    p->host_valid = false;
    return BIFEAT_OK;
}

int bifeat_fit_update(bifeat_params *p, const void *chunk, int32_t dtype, int64_t rows,
                      void *stream) {
    if (!p || !dtype_ok(dtype) || rows < 0 || (rows > 0 && !chunk)) return BIFEAT_EINVAL;
    if (p->scheme.kind == BIFEAT_VQ && !p->vq_seeded && p->fit_open && rows > 0 &&
        rows < p->scheme.vq_length)
        return BIFEAT_EINVAL;  // the first sample chunk seeds `length` entries
    if (p->scheme.kind == BIFEAT_VQ && !p->fit_open && rows > 0 && rows < p->scheme.vq_length)
        return BIFEAT_EINVAL;
    if (!p->fit_open) {
        int rc = bifeat_fit_reset(p, stream);
        if (rc) return rc;
    }
    if (rows == 0) return BIFEAT_OK;
    if (p->scheme.kind == BIFEAT_VQ) {
        BF_HIP(bf::launch_vq_train(p, chunk, dtype, rows, !p->vq_seeded, p->opt_vq_iters,
                                   (hipStream_t)stream));
        p->vq_seeded = true;
        p->vq_last_rows = rows;
        p->vq_last_rounds = p->opt_vq_iters;
        p->fit_rows += rows;
        return BIFEAT_OK;
    }
    if (p->scheme.kind == BIFEAT_SQ_LOG && p->clip_fraction > 0.0) {
        BF_HIP(bf::launch_log_hist_update(p, chunk, dtype, rows, (hipStream_t)stream));
        if (p->fit_pass == 0) p->fit_rows += rows;
        return BIFEAT_OK;
    }
    BF_HIP(bf::launch_fit_update(p, chunk, dtype, rows, (hipStream_t)stream));
    p->fit_rows += rows;
    return BIFEAT_OK;
}

int bifeat_fit_set_log_clip(bifeat_params *p, double fraction) {
    if (!p || p->scheme.kind != BIFEAT_SQ_LOG || !(fraction >= 0.0) || !(fraction < 0.5) || p->fit_open)
        return BIFEAT_EINVAL;
    p->clip_fraction = fraction;
    return BIFEAT_OK;
}

int bifeat_fit_finalize(bifeat_params *p, void *stream) {
    if (!p) return BIFEAT_EINVAL;
    if (!p->fit_open || p->fit_rows == 0) return BIFEAT_ENOTFIT;
    if (p->scheme.kind == BIFEAT_VQ) {
        p->host_valid = false;  // codebooks live on the device until asked for
        if (p->scheme.vq_metric == BIFEAT_VQ_COSINE) {
            // the encoder's entry norms come from the host, as for injected codebooks
            int rc = sync_codebooks_host(p);
            if (!rc) rc = upload_rnorm(p);
            if (rc) return rc;
        }
    } else if (p->scheme.kind == BIFEAT_SQ_UNIFORM) {
        BF_HIP(bf::launch_finalize_uniform(p, (hipStream_t)stream));
        p->host_valid = false;
    } else if (p->clip_fraction > 0.0) {
        return finalize_log_clipped(p, (hipStream_t)stream);
    } else {
        uint32_t st[2];
        BF_HIP(hipMemcpyAsync(st, p->d_fit, sizeof(st), hipMemcpyDeviceToHost, (hipStream_t)stream));
        BF_HIP(hipStreamSynchronize((hipStream_t)stream));
        float mmin, mmax;
        memcpy(&mmin, &st[0], 4);
        memcpy(&mmax, &st[1], 4);
        if (!(mmax > 0.0f)) {  // all-zero table
            p->e_min = p->e_max = 0.0;
        } else {
            p->e_min = log2((double)mmin);
            p->e_max = log2((double)mmax);
        }
        build_log_tables(p);
        int rc = upload_log(p);
        if (rc) return rc;
        p->host_valid = true;
    }
    p->fit_open = false;
    p->fitted = true;
    return BIFEAT_OK;
}

int bifeat_params_set_uniform(bifeat_params *p, const float *mn, const float *mx) {
    if (!p || !mn || !mx || p->scheme.kind != BIFEAT_SQ_UNIFORM) return BIFEAT_EINVAL;
    const size_t D = (size_t)p->D;
    for (size_t j = 0; j < D; j++)
        if (!(mn[j] <= mx[j])) return BIFEAT_EINVAL;
    p->h_min.assign(mn, mn + D);
    p->h_max.assign(mx, mx + D);
    p->h_scale.resize(D);
    p->h_inv.resize(D);
    const double L = (double)((1u << p->scheme.bits) - 1u);
    for (size_t j = 0; j < D; j++) {
        if (p->h_min[j] == 0.0f) p->h_min[j] = 0.0f;
        if (p->h_max[j] == 0.0f) p->h_max[j] = 0.0f;
        const double range = (double)p->h_max[j] - (double)p->h_min[j];
        p->h_scale[j] = range > 0.0 ? (float)(range / L) : 0.0f;
        p->h_inv[j] = range > 0.0 ? (float)(L / range) : 0.0f;
    }
    int rc = ensure_device(p);
    if (rc) return rc;
    BF_HIP(hipMemcpy(p->d_min, p->h_min.data(), 4 * D, hipMemcpyHostToDevice));
    BF_HIP(hipMemcpy(p->d_max, p->h_max.data(), 4 * D, hipMemcpyHostToDevice));
    BF_HIP(hipMemcpy(p->d_scale, p->h_scale.data(), 4 * D, hipMemcpyHostToDevice));
    BF_HIP(hipMemcpy(p->d_inv, p->h_inv.data(), 4 * D, hipMemcpyHostToDevice));
    p->host_valid = true;
    p->fitted = true;
    p->fit_open = false;
    return BIFEAT_OK;
}

int bifeat_params_get_uniform(bifeat_params *p, float *mn, float *mx, float *scale, float *inv) {
    if (!p || p->scheme.kind != BIFEAT_SQ_UNIFORM) return BIFEAT_EINVAL;
    if (!p->fitted) return BIFEAT_ENOTFIT;
    int rc = sync_uniform_host(p);
    if (rc) return rc;
    const size_t n = 4 * (size_t)p->D;
    if (mn) memcpy(mn, p->h_min.data(), n);
    if (mx) memcpy(mx, p->h_max.data(), n);
    if (scale) memcpy(scale, p->h_scale.data(), n);
    if (inv) memcpy(inv, p->h_inv.data(), n);
    return BIFEAT_OK;
}

int bifeat_params_set_log(bifeat_params *p, double e_min, double e_max) {
    if (!p || p->scheme.kind != BIFEAT_SQ_LOG || !(e_min <= e_max) || !isfinite(e_min) ||
        !isfinite(e_max))
        return BIFEAT_EINVAL;
    p->e_min = e_min;
    p->e_max = e_max;
    build_log_tables(p);
    int rc = upload_log(p);
    if (rc) return rc;
    p->host_valid = true;
    p->fitted = true;
    p->fit_open = false;
    return BIFEAT_OK;
}

int bifeat_params_get_log(bifeat_params *p, double *e_min, double *e_max, float *T, float *V) {
    if (!p || p->scheme.kind != BIFEAT_SQ_LOG) return BIFEAT_EINVAL;
    if (!p->fitted) return BIFEAT_ENOTFIT;
    if (e_min) *e_min = p->e_min;
    if (e_max) *e_max = p->e_max;
    if (T && !p->h_T.empty()) memcpy(T, p->h_T.data(), 4 * p->h_T.size());
    if (V) memcpy(V, p->h_V.data(), 4 * p->h_V.size());
    return BIFEAT_OK;
}

int bifeat_params_set_codebooks(bifeat_params *p, const float *codebooks) {
    if (!p || !codebooks || p->scheme.kind != BIFEAT_VQ) return BIFEAT_EINVAL;
    const size_t n = (size_t)p->P * p->scheme.vq_length * p->scheme.vq_width;
    p->h_cb.assign(codebooks, codebooks + n);
    int rc = ensure_device(p);
    if (rc) return rc;
    BF_HIP(hipMemcpy(p->d_cb, p->h_cb.data(), 4 * n, hipMemcpyHostToDevice));
    rc = upload_rnorm(p);
    if (rc) return rc;
    p->host_valid = true;
    p->fitted = true;
    return BIFEAT_OK;
}

int bifeat_params_get_codebooks(bifeat_params *p, float *codebooks) {
    if (!p || p->scheme.kind != BIFEAT_VQ) return BIFEAT_EINVAL;
    if (!p->fitted) return BIFEAT_ENOTFIT;
    int rc = sync_codebooks_host(p);
    if (rc) return rc;
    if (codebooks) memcpy(codebooks, p->h_cb.data(), 4 * p->h_cb.size());
    return BIFEAT_OK;
}

int bifeat_vq_distortion(bifeat_params *p, float *out, int32_t n) {
    if (!p || p->scheme.kind != BIFEAT_VQ || !out || n < 0) return BIFEAT_EINVAL;
    if (!p->vq_seeded || p->vq_last_rows == 0) return BIFEAT_ENOTFIT;
    float tmp[64];
    BF_HIP(hipDeviceSynchronize());
    BF_HIP(hipMemcpy(tmp, p->d_dist, sizeof(tmp), hipMemcpyDeviceToHost));
    for (int k = 0; k < n; k++)
        out[k] = k < p->vq_last_rounds ? tmp[k] / (float)p->vq_last_rows : 0.0f;
    return BIFEAT_OK;
}

int bifeat_quantize(bifeat_params *p, const void *chunk, int32_t dtype, int64_t rows,
                    uint8_t *codes, int64_t row0, void *stream) {
    if (!p || !dtype_ok(dtype) || rows < 0 || row0 < 0) return BIFEAT_EINVAL;
    if (rows > 0 && (!chunk || !codes)) return BIFEAT_EINVAL;
    if ((uintptr_t)codes % 16) return BIFEAT_EINVAL;
    if (!p->fitted) return BIFEAT_ENOTFIT;
    if (rows == 0) return BIFEAT_OK;
    BF_HIP(bf::launch_quantize(p, chunk, dtype, rows, codes + row0 * p->rb, (hipStream_t)stream));
    return BIFEAT_OK;
}

int bifeat_produce_fit_begin(bifeat_params *p, void *stream) {
    if (!p) return BIFEAT_EINVAL;
    if (p->scheme.kind == BIFEAT_VQ || (p->scheme.kind == BIFEAT_SQ_LOG && p->clip_fraction > 0.0))
        return BIFEAT_ENOTSUP;
    if (!p->fit_open) return bifeat_fit_reset(p, stream);
    return BIFEAT_OK;
}

int bifeat_produce_fit_end(bifeat_params *p, int64_t rows) {
    if (!p || rows < 0 || !p->fit_open) return BIFEAT_EINVAL;
    p->fit_rows += rows;
    return BIFEAT_OK;
}

int bifeat_produce_quantize_check(bifeat_params *p, const uint8_t *codes, int64_t rows, int64_t row0) {
    if (!p || rows < 0 || row0 < 0 || (rows > 0 && !codes) || (uintptr_t)codes % 16) return BIFEAT_EINVAL;
    if (p->scheme.kind == BIFEAT_VQ) return BIFEAT_ENOTSUP;
    if (!p->fitted) return BIFEAT_ENOTFIT;
    return BIFEAT_OK;
}

namespace {
// option "validate": the caller's index contract checked on the GPU before the gather
int check_inputs(bifeat_params *p, const int64_t *idx, int64_t M, int64_t N, const int64_t *indptr,
                 int64_t V, int64_t E, hipStream_t s) {
    if (!p->opt_validate) return BIFEAT_OK;
    int rc = ensure_device(p);
    if (rc) return rc;
    int32_t *d_bad = reinterpret_cast<int32_t *>(p->d_zero + 64);  // word after the zero row
    // a promised bound on the list lengths (option mean_max_degree) is part of the contract
    bf::launch_validate(idx, M, N, indptr, V, E, indptr ? p->opt_mean_max_degree : 0, d_bad, s);
    int32_t bad = 0;
    BF_HIP(hipMemcpyAsync(&bad, d_bad, sizeof(bad), hipMemcpyDeviceToHost, s));
    BF_HIP(hipStreamSynchronize(s));
    return bad ? BIFEAT_EINVAL : BIFEAT_OK;
}
}  // namespace

int bifeat_gather_codes(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *idx,
                        int64_t M, uint8_t *out, void *stream) {
    if (!p || M < 0 || N < 0) return BIFEAT_EINVAL;
    if (M > 0 && (!codes || !idx || !out || N == 0)) return BIFEAT_EINVAL;
    if ((uintptr_t)codes % 16 || (uintptr_t)out % 16) return BIFEAT_EINVAL;
    if (M == 0) return BIFEAT_OK;
    if (int rc = check_inputs(p, idx, M, N, nullptr, 0, 0, (hipStream_t)stream)) return rc;
    BF_HIP(bf::launch_gather_codes(p, codes, idx, M, out, (hipStream_t)stream));
    return BIFEAT_OK;
}

int bifeat_gather_dequant(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *idx,
                          int64_t M, float *out, void *stream) {
    if (!p || M < 0 || N < 0) return BIFEAT_EINVAL;
    if (M > 0 && (!codes || !idx || !out || N == 0)) return BIFEAT_EINVAL;
    if ((uintptr_t)codes % 16 || (uintptr_t)out % 4) return BIFEAT_EINVAL;
    if (!p->fitted) return BIFEAT_ENOTFIT;
    if (M == 0) return BIFEAT_OK;
    if (int rc = check_inputs(p, idx, M, N, nullptr, 0, 0, (hipStream_t)stream)) return rc;
    BF_HIP(bf::launch_gather_dequant(p, codes, idx, M, out, (hipStream_t)stream));
    return BIFEAT_OK;
}

int bifeat_gather_dequant_static(bifeat_params *p, const uint8_t *codes, int64_t N,
                                 const int64_t *idx, int64_t M, float *out, void *stream) {
    if (!p || M < 0 || N < 0) return BIFEAT_EINVAL;
    if (M > 0 && (!codes || !idx || !out || N == 0)) return BIFEAT_EINVAL;
    if ((uintptr_t)codes % 16 || (uintptr_t)out % 4) return BIFEAT_EINVAL;
    if (!p->fitted) return BIFEAT_ENOTFIT;  // fitted parameters already live on the device
    if (p->opt_validate) return BIFEAT_ENOTSUP;  // the checker synchronises: not for these callers
    if (M == 0) return BIFEAT_OK;
    uint32_t *planes = nullptr;
    if (p->scheme.kind == BIFEAT_VQ) {
        // only the vector-code kernels use a workspace: theirs is the static array here
        if (bf::vq_gather_scratch_bytes(p, M) > bf::static_scratch_bytes()) {
            g_hip_error = "bifeat_gather_dequant_static: request needs " +
                          std::to_string(bf::vq_gather_scratch_bytes(p, M)) + " bytes of workspace, the static one holds " +
                          std::to_string(bf::static_scratch_bytes());
            return BIFEAT_ELIMIT;
        }
        uint8_t *ptr = nullptr;
        BF_HIP(bf::static_scratch_ptr(&ptr));
        planes = (uint32_t *)ptr;
    }
    BF_HIP(bf::launch_gather_dequant(p, codes, idx, M, out, (hipStream_t)stream, planes));
    return BIFEAT_OK;
}

namespace {
int gather_aggregate(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *indptr,
                     const void *indices, bool idx32, int64_t V, int64_t E, int agg_sum, float *out,
                     void *stream) {
    if (!p || V < 0 || N < 0 || E < 0) return BIFEAT_EINVAL;
    if (V > 0 && (!codes || !indptr || !out || (E > 0 && !indices))) return BIFEAT_EINVAL;
    if ((uintptr_t)codes % 16 || (uintptr_t)out % 4) return BIFEAT_EINVAL;
    if (idx32 && N > (int64_t)INT32_MAX) return BIFEAT_EINVAL;  // row ids would not fit
    if (!p->fitted) return BIFEAT_ENOTFIT;
    // a promise broken in an earlier call (its kernel has finished since) is reported now
    if (take_status(p)) return BIFEAT_EINVAL;
    if (V == 0) return BIFEAT_OK;
    if (p->opt_validate) {
        if (idx32) return BIFEAT_ENOTSUP;  // the checker reads 64-bit entries
        if (int rc = check_inputs(p, (const int64_t *)indices, E, N, indptr, V, E, (hipStream_t)stream))
            return rc;
    }
    int rc = ensure_device(p);
    if (rc) return rc;
    const bf::MeanCall c{codes, N, indptr, indices, idx32, V, E, out, agg_sum, p->opt_mean_max_degree,
                         p->d_status, (hipStream_t)stream};
    BF_HIP(bf::launch_gather_mean(p, c));
    return BIFEAT_OK;
}
}  // namespace

int bifeat_gather_mean(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *indptr,
                       const int64_t *indices, int64_t V, int64_t E, float *out, void *stream) {
    return gather_aggregate(p, codes, N, indptr, indices, false, V, E, 0, out, stream);
}

int bifeat_gather_sum(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *indptr,
                      const int64_t *indices, int64_t V, int64_t E, float *out, void *stream) {
    return gather_aggregate(p, codes, N, indptr, indices, false, V, E, 1, out, stream);
}

int bifeat_gather_mean_i32(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *indptr,
                           const int32_t *indices, int64_t V, int64_t E, float *out, void *stream) {
    return gather_aggregate(p, codes, N, indptr, indices, true, V, E, 0, out, stream);
}

int bifeat_gather_sum_i32(bifeat_params *p, const uint8_t *codes, int64_t N, const int64_t *indptr,
                          const int32_t *indices, int64_t V, int64_t E, float *out, void *stream) {
    return gather_aggregate(p, codes, N, indptr, indices, true, V, E, 1, out, stream);
}

int bifeat_gather_mean_2hop(bifeat_params *p, const uint8_t *codes, int64_t N,
                            const int64_t *indptr1, const int64_t *indices1, int64_t V1, int64_t E1,
                            const int64_t *indptr2, const int64_t *indices2, int64_t V2, int64_t E2,
                            float *out, void *stream) {
    if (!p || N < 0 || V1 < 0 || E1 < 0 || V2 < 0 || E2 < 0) return BIFEAT_EINVAL;
    if (V2 > 0 && (!codes || !indptr2 || !out || (E2 > 0 && (!indices2 || !indptr1 || V1 == 0)) ||
                   (E1 > 0 && !indices1)))
        return BIFEAT_EINVAL;
    if ((uintptr_t)codes % 16 || (uintptr_t)out % 4) return BIFEAT_EINVAL;
    if (!p->fitted) return BIFEAT_ENOTFIT;
    if (take_status(p)) return BIFEAT_EINVAL;
    if (V2 == 0) return BIFEAT_OK;
    if (p->opt_validate) {
        if (int rc = check_inputs(p, indices1, E1, N, indptr1, V1, E1, (hipStream_t)stream)) return rc;
        if (int rc = check_inputs(p, indices2, E2, V1, indptr2, V2, E2, (hipStream_t)stream)) return rc;
    }
    int rc = ensure_device(p);
    if (rc) return rc;
    const bf::HopCall c{codes, N, indptr1, indices1, V1, E1, indptr2, indices2, V2, E2, out,
                        p->opt_mean_max_degree, p->d_status, (hipStream_t)stream};
    BF_HIP(bf::launch_gather_mean_2hop(p, c));
    return BIFEAT_OK;
}

int bifeat_poll_status(bifeat_params *p, void *stream, int32_t wait) {
    if (!p) return BIFEAT_EINVAL;
    if (wait) BF_HIP(hipStreamSynchronize((hipStream_t)stream));
    return take_status(p) ? BIFEAT_EINVAL : BIFEAT_OK;
}

int bifeat_reserve(bifeat_params *p, int64_t max_requests, void *stream) {
    if (!p || max_requests < 0) return BIFEAT_EINVAL;
    if (p->scheme.kind != BIFEAT_VQ || max_requests == 0) return BIFEAT_OK;  // no workspace needed
    int rc = ensure_device(p);
    if (rc) return rc;
    if (!bf::ensure_scratch(p, bf::vq_gather_scratch_bytes(p, max_requests), (hipStream_t)stream))
        return hip_fail(hipErrorOutOfMemory, "bifeat_reserve");
    return BIFEAT_OK;
}

int bifeat_aggregate_rows(const float *x, int64_t N, int64_t D, const int64_t *indptr,
                          const int64_t *indices, int64_t V, int64_t E, int32_t sum, float *out,
                          void *stream) {
    if (V < 0 || N < 0 || E < 0 || D <= 0 || D > (int64_t)1 << 24) return BIFEAT_EINVAL;
    if (V > 0 && (!indptr || !out || (E > 0 && (!indices || !x || N == 0)))) return BIFEAT_EINVAL;
    if ((uintptr_t)x % 4 || (uintptr_t)out % 4) return BIFEAT_EINVAL;
    if (V == 0) return BIFEAT_OK;
    BF_HIP(bf::launch_aggregate_rows(x, D, indptr, indices, V, E, sum != 0, out, (hipStream_t)stream));
    return BIFEAT_OK;
}

int bifeat_check_lists(const int64_t *indptr, const int64_t *indices, int64_t V, int64_t E,
                       int64_t N, void *stream) {
    if (V < 0 || E < 0 || N < 0 || (E > 0 && !indices) || (V > 0 && !indptr)) return BIFEAT_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    void *blk = nullptr;
    if (int rc = pool_take(&blk)) return rc;
    int32_t *d_bad = (int32_t *)blk, bad = 0;
    bf::launch_validate(indices, E, N, indptr, indptr ? V : 0, E, 0, d_bad, s);
    hipError_t e = hipMemcpyAsync(&bad, d_bad, sizeof(bad), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    pool_give(blk);
    if (e != hipSuccess) return hip_fail(e, "bifeat_check_lists");
    return bad ? BIFEAT_EINVAL : BIFEAT_OK;
}

int bifeat_scale_profile(const float *x, int64_t N, int64_t D, const int64_t *indptr,
                         const int64_t *indices, int64_t E, int32_t layers, float *work,
                         double *scale, void *stream) {
    if (N < 0 || E < 0 || D <= 0 || D > (int64_t)1 << 24 || layers < 0 || layers > 64 || !scale)
        return BIFEAT_EINVAL;
    if (N > 0 && (!x || !indptr || (E > 0 && !indices) || (layers > 0 && !work))) return BIFEAT_EINVAL;
    if ((uintptr_t)x % 4 || (uintptr_t)work % 4) return BIFEAT_EINVAL;
    if (N == 0) {
        for (int l = 0; l <= layers; l++) scale[l] = 0.0;
        return BIFEAT_OK;
    }
    hipStream_t s = (hipStream_t)stream;
    // layers+1 sums, then the flag of the index check (a pooled block holds 128 doubles)
    void *blk = nullptr;
    if (int rc = pool_take(&blk)) return rc;
    double *d_acc = (double *)blk;
    double h_acc[66];
    int32_t bad = 0;
    int32_t *d_bad = reinterpret_cast<int32_t *>(d_acc + layers + 1);
    bf::launch_zero_doubles(d_acc, layers + 2, s);
    bf::launch_validate(indices, E, N, indptr, N, E, 0, d_bad, s);
    hipError_t e = hipMemcpyAsync(&bad, d_bad, sizeof(bad), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess && !bad) {
        e = bf::launch_row_length_sum(x, N, D, d_acc, s);
        const float *src = x;
        for (int l = 1; l <= layers && e == hipSuccess; l++) {
            float *dst = work + (size_t)((l - 1) & 1) * (size_t)N * (size_t)D;
            e = bf::launch_aggregate_rows(src, D, indptr, indices, N, E, 0, dst, s);
            if (e == hipSuccess) e = bf::launch_row_length_sum(dst, N, D, d_acc + l, s);
            src = dst;
        }
        if (e == hipSuccess)
            e = hipMemcpyAsync(h_acc, d_acc, sizeof(double) * (size_t)(layers + 1),
                               hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
    }
    // the block goes back only when no work that uses it can still be running
    if (e == hipSuccess) pool_give(blk);
    if (e != hipSuccess) return hip_fail(e, "bifeat_scale_profile");
    if (bad) return BIFEAT_EINVAL;
    for (int l = 0; l <= layers; l++) scale[l] = h_acc[l] / (double)N;
    return BIFEAT_OK;
}

const char *bifeat_strerror(int status) {
    switch (status) {
        case BIFEAT_OK: return "ok";
        case BIFEAT_EINVAL: return "invalid argument";
        case BIFEAT_ENOTFIT: return "quantizer parameters not fitted";
        case BIFEAT_EHIP: return g_hip_error.empty() ? "HIP error" : g_hip_error.c_str();
        case BIFEAT_ENOTSUP: return "not supported";
        case BIFEAT_ELIMIT:
            return g_hip_error.empty() ? "request exceeds a fixed limit of the library" : g_hip_error.c_str();
        default: return "unknown status";
    }
}

}  // extern "C"
