// C ABI of libhdc: argument checking, the context (device copies of the tables laid out for
// the kernels, scratch buffers) and dispatch to the kernel launchers.  No compute here.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "bit_spread.h"
#include "hdc_internal.h"

namespace hdc {

static thread_local char g_hip_err[256] = "";

int hip_fail(hipError_t e, const char *what) {
    snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s", what, hipGetErrorString(e));
    (void)hipGetLastError();   // clear the sticky error so later calls report their own
    return HDC_EHIP;
}

constexpr int64_t kEncodeChunk = 65536;      // samples quantised per encode launch
constexpr int64_t kPermRows = 1 << 22;       // rows grouped by class per training launch

static void free_ctx(hdc_ctx_impl *c) {
    if (!c) return;
    void *ptrs[] = {c->item_d, c->level_d, c->tie_d, c->lo_d, c->scale_d, c->q_d, c->cls_cnt_d,
                    c->cls_off_d, c->cls_cur_d, c->cls_blk_d, c->perm_d, c->partial_d, c->ob_part_d, c->ob_wts_d, c->ob_norm_d,
                    c->ob_col_d, c->ob_carry_d, c->ob_coef_d, c->ob_share_d, c->on_bits_d, c->ob_ln_d, c->ob_lw_d, c->ob_meta_d,
                    c->citem_d, c->clevel_d, c->hvc_d, c->expand_d,
                    c->sp_b_d, c->sp_e_d, c->sp_base_d, c->sp_fb_d, c->sp_blocks_d,
                    c->ct_tau_d[0], c->ct_col_d[0], c->ct_k_d[0], c->ct_bt_d[0],
                    c->ct_tau_d[1], c->ct_col_d[1], c->ct_k_d[1], c->ct_bt_d[1],
                    c->ct_tau_d[2], c->ct_col_d[2], c->ct_k_d[2], c->ct_bt_d[2],
                    c->wd_items_d, c->wd_bx_d, c->wd_src_d, c->bad_labels_d};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    for (int k = 0; k < HDC_K_COUNT; ++k) {
        if (!c->prof_ev[k]) continue;
        for (int i = 0; i < 2 * HDC_PROFILE_SLOTS; ++i)
            if (c->prof_ev[k][i]) (void)hipEventDestroy(c->prof_ev[k][i]);
        free(c->prof_ev[k]);
    }
    delete c;
}

template <typename T>
static int dev_alloc(T **p, size_t count) {
    hipError_t e = hipMalloc(reinterpret_cast<void **>(p), count * sizeof(T) + 256);
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        return HDC_ENOMEM;
    }
    if (e != hipSuccess) return hip_fail(e, "hipMalloc");
    return HDC_OK;
}

static bool pads_are_zero(const uint32_t *t, int64_t rows, int W, uint32_t last_mask) {
    for (int64_t r = 0; r < rows; ++r)
        if (t[r * W + (W - 1)] & ~last_mask) return false;
    return true;
}

// ---- level-invariant dimensions: host-side preparation ---------------------------------------
// Word w of row r in the slice-major device layout [Wp / 64][rows][64].
static inline size_t slice_major(int rows, int r, int w) {
    return ((size_t)(w / kSliceWords) * rows + r) * kSliceWords + (w % kSliceWords);
}

constexpr int64_t kCompactMaxBits = 200000000;   // table bits the host is willing to repack at create

// Builds the spreading table and the constant bits of the level-invariant dimensions (the latter
// by encoding one sample with the full tables: at an invariant dimension every sample gives the
// same bit), decides whether the vector kernels encode the varying dimensions only and, if so,
// builds the compact tables.  Leaves c->compact false (and, before the table is up, c->expand_d
// null) on any doubt; only a failed allocation or copy is an error.
static int prepare_compact(hdc_ctx_impl *c, const uint32_t *item, const uint32_t *level, const uint32_t *tie) {
    const hdc_params &p = c->p;
    const int W = c->W;
    c->compact = false;
    if (((int64_t)c->Fp + p.L) * p.D > kCompactMaxBits) return HDC_OK;
    std::vector<uint32_t> keep((size_t)W, 0u);   // bit set = some level vector differs from level 0 there
    int64_t varying = 0;
    for (int w = 0; w < W; ++w) {
        uint32_t diff = 0;
        for (int l = 1; l < p.L; ++l) diff |= level[(size_t)l * W + w] ^ level[w];
        keep[w] = diff;
        varying += __builtin_popcount(diff);
    }
    const int Wc = (int)((varying + 31) / 32);
    const int Wcp = (Wc + kSliceWords - 1) / kSliceWords * kSliceWords;

    // spreading table, checked against the definition before it is trusted
    std::vector<uint32_t> tab((size_t)8 * W, 0u);
    uint32_t off = 0;
    for (int w = 0; w < W; ++w) {
        uint32_t stage[5];
        spread_stages(keep[w], stage);
        const uint32_t probes[3] = {0xffffffffu, 0x55555555u, 0x9e3779b9u};
        for (uint32_t x : probes) {
            uint32_t want = 0;
            int j = 0;
            for (uint32_t m = keep[w]; m; m &= m - 1, ++j) want |= ((x >> j) & 1u) << __builtin_ctz(m);
            if (spread_bits(x, keep[w], stage) != want) return HDC_OK;   // never expected; keeps the full path
        }
        tab[w] = off;
        tab[(size_t)W + w] = keep[w];
        for (int i = 0; i < 5; ++i) tab[(size_t)(2 + i) * W + w] = stage[i];
        off += (uint32_t)__builtin_popcount(keep[w]);
    }

    // constant bits: one sample (all features zero) through the full tables
    {
        const size_t esz = p.feat_dtype == HDC_U8 ? 1 : 4;
        void *x_d = nullptr;
        uint32_t *h_d = nullptr;
        std::vector<uint32_t> h((size_t)W);
        hipError_t e = hipMalloc(&x_d, (size_t)p.F * esz + 256);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&h_d), (size_t)W * 4 + 256);
        if (e == hipSuccess) e = hipMemset(x_d, 0, (size_t)p.F * esz);
        int rc = e == hipSuccess ? launch_encode(c, x_d, 1, h_d, nullptr) : HDC_EHIP;
        if (rc == HDC_OK) e = hipMemcpy(h.data(), h_d, (size_t)W * 4, hipMemcpyDeviceToHost);
        if (x_d) (void)hipFree(x_d);
        if (h_d) (void)hipFree(h_d);
        if (e == hipErrorOutOfMemory) {
            (void)hipGetLastError();
            return HDC_ENOMEM;
        }
        if (e != hipSuccess) return hip_fail(e, "constant bits of the level-invariant dimensions");
        if (rc != HDC_OK) return rc;
        for (int w = 0; w < W; ++w) tab[(size_t)7 * W + w] = h[w] & ~keep[w];
    }

    // The table is kept in any case (the contraction encoders take the constant bits from it).
    int rc = dev_alloc(&c->expand_d, tab.size());
    if (rc != HDC_OK) return rc;
    hipError_t e = hipMemcpy(c->expand_d, tab.data(), tab.size() * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpy");
    if (varying * 4 > (int64_t)p.D * 3) return HDC_OK;   // less than a quarter to gain: not worth a second pass of the vector kernels
    // compact tables in the same padded slice-major layout as the full ones
    if (Wc > 0) {
        std::vector<uint32_t> item_h((size_t)c->Fp * Wcp, 0u), level_h((size_t)p.L * Wcp, 0u);
        std::vector<uint32_t> row((size_t)W), crow((size_t)Wc);
        auto put = [&](std::vector<uint32_t> &dst, int rows, int r, const uint32_t *src_row) {
            std::fill(crow.begin(), crow.end(), 0u);
            compact_row(src_row, keep.data(), W, crow.data());
            for (int w = 0; w < Wc; ++w) dst[slice_major(rows, r, w)] = crow[w];
        };
        for (int l = 0; l < p.L; ++l) put(level_h, p.L, l, level + (size_t)l * W);
        for (int f = 0; f < c->Fp; ++f) {
            if (f < p.F) {
                put(item_h, c->Fp, f, item + (size_t)f * W);
            } else if (f == p.F && c->votes != p.F) {
                for (int w = 0; w < W; ++w) row[w] = tie[w] ^ level[w];
                put(item_h, c->Fp, f, row.data());
            } else {
                put(item_h, c->Fp, f, level);
            }
        }
        rc = dev_alloc(&c->citem_d, item_h.size());
        if (rc == HDC_OK) rc = dev_alloc(&c->clevel_d, level_h.size());
        if (rc == HDC_OK) rc = dev_alloc(&c->hvc_d, (size_t)c->q_rows * Wc);
        if (rc != HDC_OK) return rc;
        e = hipMemcpy(c->citem_d, item_h.data(), item_h.size() * 4, hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(c->clevel_d, level_h.data(), level_h.size() * 4, hipMemcpyHostToDevice);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpy");
    }
    c->Wc = Wc;
    c->Wcp = Wcp;
    c->compact = true;
    return HDC_OK;
}

static int create(hdc_ctx **out, const hdc_params *p, const uint32_t *item, const uint32_t *level,
                  const uint32_t *tie, const float *lo, const float *scale) {
    if (!out) return HDC_EINVAL;
    *out = nullptr;
    if (!p || !item || !level || !tie) return HDC_EINVAL;
    if (p->D < 1 || p->D > HDC_MAX_D || p->F < 1 || p->F > HDC_MAX_F || p->L < 1 ||
        p->L > HDC_MAX_L || p->C < 1 || p->C > HDC_MAX_C)
        return HDC_EINVAL;
    if (p->feat_dtype == HDC_F32) {
        if (!lo || !scale) return HDC_EINVAL;
    } else if (p->feat_dtype == HDC_U8) {
        if (lo || scale) return HDC_EINVAL;
    } else {
        return HDC_EINVAL;
    }
    const int W = (p->D + 31) / 32;
    const uint32_t last_mask = (p->D & 31) ? ((1u << (p->D & 31)) - 1u) : 0xffffffffu;
    if (!pads_are_zero(item, p->F, W, last_mask) || !pads_are_zero(level, p->L, W, last_mask) ||
        !pads_are_zero(tie, 1, W, last_mask))
        return HDC_EINVAL;

    hdc_ctx_impl *c = new (std::nothrow) hdc_ctx_impl();
    if (!c) return HDC_ENOMEM;
    memset(c, 0, sizeof(*c));
    c->p = *p;
    c->W = W;
    c->Wp = (W + kSliceWords - 1) / kSliceWords * kSliceWords;
    c->votes = (p->F & 1) ? p->F : p->F + 1;
    c->Fp = (c->votes + kFeatBlock - 1) / kFeatBlock * kFeatBlock;
    c->last_word_mask = last_mask;
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) {
        delete c;
        return hip_fail(e, "hipGetDevice");
    }
    e = hipDeviceGetAttribute(&c->num_cus, hipDeviceAttributeMultiprocessorCount, c->device);
    if (e != hipSuccess || c->num_cus < 1) {
        delete c;
        return hip_fail(e, "hipDeviceGetAttribute");
    }

    // Host staging of the padded device tables (layout described in hdc_internal.h).
    std::vector<uint32_t> item_h, level_h, tie_h;
    try {
        item_h.assign((size_t)c->Fp * c->Wp, 0u);
        level_h.assign((size_t)p->L * c->Wp, 0u);
        tie_h.assign((size_t)c->Wp, 0u);
    } catch (const std::bad_alloc &) {
        delete c;
        return HDC_ENOMEM;
    }
    // slice-major layout: word w of row r lives at [(w / 64) * rows + r][w % 64]
    const int nsl = c->Wp / kSliceWords;
    auto put = [&](std::vector<uint32_t> &dst, int rows, int r, const uint32_t *src_row) {
        for (int w = 0; w < W; ++w)
            dst[((size_t)(w / kSliceWords) * rows + r) * kSliceWords + (w % kSliceWords)] = src_row[w];
    };
    (void)nsl;
    std::vector<uint32_t> tmp((size_t)W);
    for (int l = 0; l < p->L; ++l) put(level_h, p->L, l, level + (size_t)l * W);
    memcpy(tie_h.data(), tie, (size_t)W * 4);
    for (int f = 0; f < c->Fp; ++f) {
        if (f < p->F) {
            put(item_h, c->Fp, f, item + (size_t)f * W);
        } else if (f == p->F && c->votes != p->F) {
            for (int w = 0; w < W; ++w) tmp[w] = tie[w] ^ level[w];   // binds with level 0 to tie
            put(item_h, c->Fp, f, tmp.data());
        } else {
            put(item_h, c->Fp, f, level);                             // binds with level 0 to zero
        }
    }

    int rc = HDC_OK;
#define TRY(x)                         \
    do {                               \
        if (rc == HDC_OK) rc = (x);    \
    } while (0)
#define TRY_HIP(x)                                              \
    do {                                                        \
        if (rc == HDC_OK) {                                     \
            hipError_t e2 = (x);                                \
            if (e2 != hipSuccess) rc = hip_fail(e2, #x);        \
        }                                                       \
    } while (0)
    TRY(dev_alloc(&c->item_d, item_h.size()));
    TRY(dev_alloc(&c->level_d, level_h.size()));
    TRY(dev_alloc(&c->tie_d, tie_h.size()));
    TRY_HIP(hipMemcpy(c->item_d, item_h.data(), item_h.size() * 4, hipMemcpyHostToDevice));
    TRY_HIP(hipMemcpy(c->level_d, level_h.data(), level_h.size() * 4, hipMemcpyHostToDevice));
    TRY_HIP(hipMemcpy(c->tie_d, tie_h.data(), tie_h.size() * 4, hipMemcpyHostToDevice));
    if (p->feat_dtype == HDC_F32) {
        TRY(dev_alloc(&c->lo_d, (size_t)p->F));
        TRY(dev_alloc(&c->scale_d, (size_t)p->F));
        TRY_HIP(hipMemcpy(c->lo_d, lo, (size_t)p->F * 4, hipMemcpyHostToDevice));
        TRY_HIP(hipMemcpy(c->scale_d, scale, (size_t)p->F * 4, hipMemcpyHostToDevice));
    }
    // rows of a chunk of the vector encoders: their scratch (2 bytes a feature here, 4 more in the
    // sparse encoder) stays within 512 MB whatever F is; the chunk loops take any count
    c->q_rows = std::max<int64_t>(64, std::min<int64_t>(kEncodeChunk, ((int64_t)512 << 20) / ((int64_t)c->Fp * 6) / 64 * 64));
    TRY(dev_alloc(&c->q_d, (size_t)c->q_rows * c->Fp));
    TRY(dev_alloc(&c->bad_labels_d, 1));
    TRY(dev_alloc(&c->cls_cnt_d, (size_t)p->C + 1));
    TRY(dev_alloc(&c->cls_off_d, (size_t)p->C + 1));
    TRY(dev_alloc(&c->cls_cur_d, (size_t)p->C + 2));
    TRY_HIP(hipMemset(c->cls_cur_d, 0, ((size_t)p->C + 2) * 4));   // (the grouping kernels leave it zero again)
    TRY(dev_alloc(&c->cls_blk_d, (size_t)p->C + 1));
    c->perm_rows = kPermRows;
    TRY(dev_alloc(&c->perm_d, (size_t)c->perm_rows));
    c->partial_items = classical_max_items(c);
    if (c->partial_items < 0 && rc == HDC_OK) rc = HDC_EHIP;
    TRY(dev_alloc(&c->partial_d, (size_t)c->partial_items * c->Wp * 16));
    TRY_HIP(hipDeviceSynchronize());
    try {
        TRY(prepare_compact(c, item, level, tie));
        TRY(prepare_contract(c, item, level, tie));
        TRY(prepare_wide(c, item, level, tie));
    } catch (const std::bad_alloc &) {
        rc = HDC_ENOMEM;
    }
    TRY_HIP(hipDeviceSynchronize());
#undef TRY
#undef TRY_HIP
    if (rc != HDC_OK) {
        free_ctx(c);
        return rc;
    }
    *out = reinterpret_cast<hdc_ctx *>(c);
    return HDC_OK;
}

__global__ __launch_bounds__(256) void count_bad_labels_kernel(const int32_t *__restrict__ labels, int64_t N, int C,
                                                               unsigned long long *bad) {
    int64_t mine = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < N; i += (int64_t)gridDim.x * 256) {
        const int y = labels[i];
        mine += (y < 0 || y >= C) ? 1 : 0;
    }
    if (mine) atomicAdd(bad, (unsigned long long)mine);
}
__global__ void zero_u64_kernel(unsigned long long *p) { *p = 0; }

int count_bad_labels(hdc_ctx_impl *c, const int32_t *labels, int64_t N, hipStream_t s, int64_t *bad) {
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, s, c->bad_labels_d);
    const int64_t blocks = std::min<int64_t>((N + 255) / 256, 4096);
    hipLaunchKernelGGL(count_bad_labels_kernel, dim3((unsigned)blocks), dim3(256), 0, s, labels, N, c->p.C,
                       c->bad_labels_d);
    unsigned long long got = 0;
    HDC_HIP(hipMemcpyAsync(&got, c->bad_labels_d, sizeof(got), hipMemcpyDeviceToHost, s));
    HDC_HIP(hipStreamSynchronize(s));
    *bad = (int64_t)got;
    return HDC_OK;
}

// HDC_ELABEL if label checking is on and a label is outside [0, C); HDC_OK otherwise.
static int labels_ok(hdc_ctx_impl *c, const int32_t *labels, int64_t N, hipStream_t s) {
    if (!c->check_labels) return HDC_OK;
    int64_t bad = 0;
    const int rc = count_bad_labels(c, labels, N, s, &bad);
    if (rc != HDC_OK) return rc;
    return bad ? HDC_ELABEL : HDC_OK;
}

static inline hdc_ctx_impl *impl(hdc_ctx *c) { return reinterpret_cast<hdc_ctx_impl *>(c); }
static inline bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }
static inline bool aligned8(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 7u) == 0; }

}  // namespace hdc

using namespace hdc;

extern "C" {

int hdc_create(hdc_ctx **out, const hdc_params *p, const uint32_t *item_host,
               const uint32_t *level_host, const uint32_t *tie_host, const float *lo_host,
               const float *scale_host) {
    return create(out, p, item_host, level_host, tie_host, lo_host, scale_host);
}

int hdc_destroy(hdc_ctx *ctx) {
    if (!ctx) return HDC_OK;
    hipError_t e = hipDeviceSynchronize();
    free_ctx(impl(ctx));
    if (e != hipSuccess) return hip_fail(e, "hipDeviceSynchronize");
    return HDC_OK;
}

int hdc_encode(hdc_ctx *ctx, const void *feats_dev, int64_t N, uint32_t *hv_dev, void *stream) {
    if (!ctx || N < 0) return HDC_EINVAL;
    if (N == 0) return HDC_OK;
    if (!feats_dev || !hv_dev || !aligned4(hv_dev)) return HDC_EINVAL;
    if (impl(ctx)->p.feat_dtype == HDC_F32 && !aligned4(feats_dev)) return HDC_EINVAL;
    return launch_encode(impl(ctx), feats_dev, N, hv_dev, static_cast<hipStream_t>(stream));
}

int hdc_encode_sparse(hdc_ctx *ctx, const void *feats_dev, int64_t N, uint32_t *hv_dev, void *stream) {
    if (!ctx || N < 0) return HDC_EINVAL;
    if (N == 0) return HDC_OK;
    if (!feats_dev || !hv_dev || !aligned4(hv_dev)) return HDC_EINVAL;
    if (impl(ctx)->p.feat_dtype == HDC_F32 && !aligned4(feats_dev)) return HDC_EINVAL;
    return launch_encode_sparse(impl(ctx), feats_dev, N, hv_dev, static_cast<hipStream_t>(stream));
}

int32_t hdc_encoded_words(const hdc_ctx *ctx) {
    if (!ctx) return -1;
    const hdc_ctx_impl *c = reinterpret_cast<const hdc_ctx_impl *>(ctx);
    return c->compact ? c->Wc : c->W;
}

int hdc_train_classical(hdc_ctx *ctx, const uint32_t *hv_dev, const int32_t *labels_dev, int64_t N,
                        int32_t *acc_dev, int64_t *class_n_dev, void *stream) {
    if (!ctx || N < 0) return HDC_EINVAL;
    if (N == 0) return HDC_OK;
    if (!hv_dev || !labels_dev || !acc_dev || !class_n_dev) return HDC_EINVAL;
    if (!aligned4(hv_dev) || !aligned4(labels_dev) || !aligned4(acc_dev) || !aligned8(class_n_dev))
        return HDC_EINVAL;
    if (const int rc = labels_ok(impl(ctx), labels_dev, N, static_cast<hipStream_t>(stream))) return rc;
    return launch_train_classical(impl(ctx), hv_dev, labels_dev, N, acc_dev, class_n_dev,
                                  static_cast<hipStream_t>(stream));
}

int hdc_binarize_classical(hdc_ctx *ctx, const int32_t *acc_dev, const int64_t *class_n_dev,
                           uint32_t *class_hv_dev, void *stream) {
    if (!ctx || !acc_dev || !class_n_dev || !class_hv_dev) return HDC_EINVAL;
    if (!aligned4(acc_dev) || !aligned8(class_n_dev) || !aligned4(class_hv_dev)) return HDC_EINVAL;
    return launch_binarize_classical(impl(ctx), acc_dev, class_n_dev, class_hv_dev,
                                     static_cast<hipStream_t>(stream));
}

int hdc_train_online(hdc_ctx *ctx, const uint32_t *hv_dev, const int32_t *labels_dev, int64_t N,
                     int32_t epochs, float lr, float *acc_dev, void *stream) {
    if (!ctx || N < 0 || epochs < 0) return HDC_EINVAL;
    if (N == 0 || epochs == 0) return HDC_OK;
    if (!hv_dev || !labels_dev || !acc_dev) return HDC_EINVAL;
    if (!aligned4(hv_dev) || !aligned4(labels_dev) || !aligned4(acc_dev)) return HDC_EINVAL;
    if (const int rc = labels_ok(impl(ctx), labels_dev, N, static_cast<hipStream_t>(stream))) return rc;
    return launch_train_online(impl(ctx), hv_dev, labels_dev, N, epochs, lr, acc_dev,
                               static_cast<hipStream_t>(stream));
}

int hdc_train_online_batched(hdc_ctx *ctx, const uint32_t *hv_dev, const int32_t *labels_dev, int64_t N,
                             int32_t epochs, float lr, int64_t batch, float *acc_dev, void *stream) {
    if (!ctx || N < 0 || epochs < 0 || batch < 1) return HDC_EINVAL;
    if (N == 0 || epochs == 0) return HDC_OK;
    if (!hv_dev || !labels_dev || !acc_dev) return HDC_EINVAL;
    if (!aligned4(hv_dev) || !aligned4(labels_dev) || !aligned4(acc_dev)) return HDC_EINVAL;
    if (const int rc = labels_ok(impl(ctx), labels_dev, N, static_cast<hipStream_t>(stream))) return rc;
    return launch_train_online_batched(impl(ctx), hv_dev, labels_dev, N, epochs, lr, batch, acc_dev,
                                       static_cast<hipStream_t>(stream));
}

int hdc_binarize_online(hdc_ctx *ctx, const float *acc_dev, uint32_t *class_hv_dev, void *stream) {
    if (!ctx || !acc_dev || !class_hv_dev) return HDC_EINVAL;
    if (!aligned4(acc_dev) || !aligned4(class_hv_dev)) return HDC_EINVAL;
    return launch_binarize_online(impl(ctx), acc_dev, class_hv_dev, static_cast<hipStream_t>(stream));
}

int hdc_search_cosine(hdc_ctx *ctx, const uint32_t *hv_dev, int64_t N, const float *acc_dev, float *cos_dev,
                      int32_t *pred_dev, void *stream) {
    if (!ctx || N < 0) return HDC_EINVAL;
    if (N == 0) return HDC_OK;
    if (!hv_dev || !acc_dev || !pred_dev) return HDC_EINVAL;
    if (!aligned4(hv_dev) || !aligned4(acc_dev) || !aligned4(cos_dev) || !aligned4(pred_dev)) return HDC_EINVAL;
    return launch_search_cosine(impl(ctx), hv_dev, N, acc_dev, cos_dev, pred_dev, static_cast<hipStream_t>(stream));
}

int hdc_pack(hdc_ctx *ctx, const uint8_t *bits_dev, int64_t N, uint32_t *hv_dev, void *stream) {
    if (!ctx || N < 0) return HDC_EINVAL;
    if (N == 0) return HDC_OK;
    if (!bits_dev || !hv_dev || !aligned4(hv_dev)) return HDC_EINVAL;
    return launch_pack(impl(ctx), bits_dev, N, hv_dev, static_cast<hipStream_t>(stream));
}

int hdc_unpack(hdc_ctx *ctx, const uint32_t *hv_dev, int64_t N, uint8_t *bits_dev, void *stream) {
    if (!ctx || N < 0) return HDC_EINVAL;
    if (N == 0) return HDC_OK;
    if (!bits_dev || !hv_dev || !aligned4(hv_dev)) return HDC_EINVAL;
    return launch_unpack(impl(ctx), hv_dev, N, bits_dev, static_cast<hipStream_t>(stream));
}

int hdc_hsum(hdc_ctx *ctx, const uint32_t *hv_dev, int64_t N, int32_t *sum_dev, void *stream) {
    if (!ctx || N < 0) return HDC_EINVAL;
    if (N == 0) return HDC_OK;
    if (!hv_dev || !sum_dev || !aligned4(hv_dev) || !aligned4(sum_dev)) return HDC_EINVAL;
    return launch_hsum(impl(ctx), hv_dev, N, sum_dev, static_cast<hipStream_t>(stream));
}

int hdc_vsum(hdc_ctx *ctx, const uint32_t *hv_dev, int64_t N, int32_t *sum_dev, void *stream) {
    if (!ctx || N < 0 || N > INT32_MAX) return HDC_EINVAL;
    if (!sum_dev || !aligned4(sum_dev) || (N > 0 && (!hv_dev || !aligned4(hv_dev)))) return HDC_EINVAL;
    return launch_vsum(impl(ctx), hv_dev, N, sum_dev, static_cast<hipStream_t>(stream));
}

int hdc_vsum_static(int32_t D, const uint32_t *hv_dev, int64_t N, int32_t *sum_dev, void *stream) {
    if (D < 1 || N < 0 || N > INT32_MAX) return HDC_EINVAL;
    if (D > 16384) return HDC_ELIMIT;
    if (!sum_dev || !aligned4(sum_dev) || (N > 0 && (!hv_dev || !aligned4(hv_dev)))) return HDC_EINVAL;
    return vsum_static(D, hv_dev, N, sum_dev, static_cast<hipStream_t>(stream));
}

int hdc_search(hdc_ctx *ctx, const uint32_t *hv_dev, int64_t N, const uint32_t *class_hv_dev,
               uint32_t *dist_dev, int32_t *pred_dev, void *stream) {
    if (!ctx || N < 0) return HDC_EINVAL;
    if (N == 0) return HDC_OK;
    if (!hv_dev || !class_hv_dev || !pred_dev) return HDC_EINVAL;
    if (!aligned4(hv_dev) || !aligned4(class_hv_dev) || !aligned4(pred_dev) || !aligned4(dist_dev))
        return HDC_EINVAL;
    return launch_search(impl(ctx), hv_dev, N, class_hv_dev, dist_dev, pred_dev,
                         static_cast<hipStream_t>(stream));
}

int hdc_set_label_check(hdc_ctx *ctx, int enable) {
    if (!ctx) return HDC_EINVAL;
    impl(ctx)->check_labels = enable != 0;
    return HDC_OK;
}

int hdc_reserve(hdc_ctx *ctx, unsigned what, int64_t max_batch, int64_t max_queries, void *stream) {
    if (!ctx || (what & ~(unsigned)HDC_RESERVE_ALL)) return HDC_EINVAL;
    if (((what & HDC_RESERVE_ONLINE_BATCHED) && max_batch < 1) || ((what & HDC_RESERVE_SEARCH_COSINE) && max_queries < 1))
        return HDC_EINVAL;
    hdc_ctx_impl *c = impl(ctx);
    int rc = HDC_OK;
    if (rc == HDC_OK && (what & HDC_RESERVE_ONLINE)) rc = reserve_online(c);
    if (rc == HDC_OK && (what & HDC_RESERVE_ONLINE_BATCHED)) rc = reserve_online_batched(c, max_batch);
    if (rc == HDC_OK && (what & HDC_RESERVE_SEARCH_COSINE)) rc = reserve_search_cosine(c, max_queries);
    if (rc == HDC_OK && (what & HDC_RESERVE_ENCODE_SPARSE)) rc = reserve_sparse(c, static_cast<hipStream_t>(stream));
    return rc;
}

int hdc_profile_enable(hdc_ctx *ctx, int enable) {
    if (!ctx) return HDC_EINVAL;
    hdc_ctx_impl *c = impl(ctx);
    if (enable) {
        for (int k = 0; k < HDC_K_COUNT; ++k) {
            if (c->prof_ev[k]) continue;
            c->prof_ev[k] = static_cast<hipEvent_t *>(calloc(2 * HDC_PROFILE_SLOTS, sizeof(hipEvent_t)));
            if (!c->prof_ev[k]) return HDC_ENOMEM;
            for (int i = 0; i < 2 * HDC_PROFILE_SLOTS; ++i) HDC_HIP(hipEventCreate(&c->prof_ev[k][i]));
        }
    }
    c->prof_on = enable != 0;
    return HDC_OK;
}

int hdc_profile_read(hdc_ctx *ctx, int kernel_id, double *total_ms, int64_t *launches) {
    if (!ctx || kernel_id < 0 || kernel_id >= HDC_K_COUNT || !total_ms || !launches) return HDC_EINVAL;
    hdc_ctx_impl *c = impl(ctx);
    double sum = 0.0;
    const int n = c->prof_ev[kernel_id] ? c->prof_used[kernel_id] : 0;
    for (int i = 0; i < n; ++i) {
        float ms = 0.0f;
        HDC_HIP(hipEventSynchronize(c->prof_ev[kernel_id][2 * i + 1]));
        HDC_HIP(hipEventElapsedTime(&ms, c->prof_ev[kernel_id][2 * i], c->prof_ev[kernel_id][2 * i + 1]));
        sum += (double)ms;
    }
    c->prof_used[kernel_id] = 0;
    *total_ms = sum;
    *launches = n;
    return HDC_OK;
}

const char *hdc_strerror(int code) {
    switch (code) {
        case HDC_OK: return "ok";
        case HDC_EINVAL: return "invalid argument";
        case HDC_ENOMEM: return "out of memory";
        case HDC_EHIP: return "HIP runtime error (see hdc_last_hip_error)";
        case HDC_ELIMIT: return "size beyond what this build supports";
        case HDC_ELABEL: return "a label is outside [0, C) (label checking is on)";
        default: return "unknown status";
    }
}

const char *hdc_last_hip_error(void) { return g_hip_err; }

const char *hdc_version(void) { return "0.1.0"; }

}  // extern "C"
