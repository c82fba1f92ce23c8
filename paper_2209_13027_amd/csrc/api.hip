// C ABI of libddcca: argument validation, scratch management and the host-side
// orchestration of the kernels.  No arithmetic of the method happens on the host.
#include <stdio.h>

#include <algorithm>
#include <new>

#include "ddcca_internal.h"

namespace ddcca {

int fail(ddcca_ctx *ctx, int code, const std::string &msg)
{
    if (ctx) ctx->err = msg;
    return code;
}

int hip_fail(ddcca_ctx *ctx, hipError_t e, const char *what)
{
    (void)hipGetLastError();   // clear the sticky (non-fatal) error state
    return fail(ctx, e == hipErrorOutOfMemory ? DDCCA_ENOMEM : DDCCA_EHIP,
                std::string(what) + ": " + hipGetErrorString(e));
}

int device_ready(ddcca_ctx *ctx)
{
    DDCCA_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->n_cu == 0) {
        int cu = 0;
        DDCCA_HIP(ctx, hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, ctx->device));
        ctx->n_cu = cu > 0 ? cu : 256;
    }
    return DDCCA_OK;
}

int ensure(ddcca_ctx *ctx, Buffer &b, size_t bytes)
{
    if (b.bytes >= bytes && b.ptr) return DDCCA_OK;
    if (b.ptr) {
        // earlier work on the stream may still use the old allocation
        DDCCA_HIP(ctx, hipStreamSynchronize(ctx->stream));
        DDCCA_HIP(ctx, hipFree(b.ptr));
        b.ptr = nullptr;
        b.bytes = 0;
    }
    size_t want = std::max<size_t>(bytes, 256);
    DDCCA_HIP(ctx, hipMalloc(&b.ptr, want));
    b.bytes = want;
    return DDCCA_OK;
}

int ensure_flags(ddcca_ctx *ctx)
{
    if (ctx->flags.ptr) return DDCCA_OK;
    int rc;
    if ((rc = ensure(ctx, ctx->flags, 4 * sizeof(int)))) return rc;
    DDCCA_HIP(ctx, hipMemsetAsync(ctx->flags.ptr, 0, 4 * sizeof(int), ctx->stream));
    return DDCCA_OK;
}

ProfScope::ProfScope(ddcca_ctx *c, int kernel_id) : ctx(c), id(kernel_id)
{
    if (!ctx->prof || !((ctx->prof_mask >> id) & 1u)) return;
    ProfSlot &s = ctx->prof_slot[id];
    if (s.used == s.start.size()) {
        hipEvent_t a = nullptr, b = nullptr;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
            ctx->prof = false;
            return;
        }
        s.start.push_back(a);
        s.stop.push_back(b);
    }
    (void)hipEventRecord(s.start[s.used], ctx->stream);
}

ProfScope::~ProfScope()
{
    if (!ctx->prof || !((ctx->prof_mask >> id) & 1u)) return;
    ProfSlot &s = ctx->prof_slot[id];
    if (s.used >= s.stop.size()) return;
    (void)hipEventRecord(s.stop[s.used], ctx->stream);
    s.used += 1;
    s.launches += 1;
}

static bool valid_k(int k) { return k >= DDCCA_MIN_K && k <= DDCCA_MAX_K && (k & 1); }

static int check_image_args(ddcca_ctx *ctx, int64_t n, int h, int w, int k)
{
    if (n < 0) return fail(ctx, DDCCA_EINVAL, "negative image count");
    if (h < 1 || w < 1) return fail(ctx, DDCCA_EINVAL, "image height and width must be >= 1");
    if ((int64_t)h * w > (int64_t)1 << 26) return fail(ctx, DDCCA_EINVAL, "image larger than 2^26 pixels");
    if (!valid_k(k)) return fail(ctx, DDCCA_EINVAL, "patch side k must be odd and in 3..9");
    return DDCCA_OK;
}

static void free_buffer(Buffer &b)
{
    if (b.ptr) (void)hipFree(b.ptr);
    b.ptr = nullptr;
    b.bytes = 0;
}

// The Gram contribution of n_maps map pairs: the dense kernel, or the lag statistics.
static int accumulate_gram(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t n_maps)
{
    if (ctx->lag_active)
        return launch_lag_gram(ctx, v1, v2, n_maps, ctx->h, ctx->w, ctx->k, (double *)ctx->lag_slots.ptr,
                               max_lag_slots(ctx), &ctx->lag_valid, (double *)ctx->lag_col_slots.ptr,
                               max_lag_col_slots(ctx), &ctx->lag_col_valid);
    return launch_patch_gram(ctx, v1, v2, n_maps, ctx->h, ctx->w, ctx->k, false, (double *)ctx->slots.ptr,
                             max_gram_slots(ctx, ctx->k), &ctx->slots_valid);
}

// lag statistics in the two slot sets -> stacked Gram
static int lag_finish(ddcca_ctx *ctx, int valid, int col_valid, double *stacked_out)
{
    const int k = ctx->k;
    int rc;
    if ((rc = launch_reduce_slots(ctx, (const double *)ctx->lag_slots.ptr, valid, (int)lag_slot_doubles(k),
                                  (double *)ctx->lag_R.ptr)))
        return rc;
    if ((rc = launch_reduce_slots(ctx, (const double *)ctx->lag_col_slots.ptr, col_valid,
                                  (int)lag_col_slot_doubles(k), (double *)ctx->lag_C.ptr)))
        return rc;
    return launch_lag_to_stacked(ctx, (const double *)ctx->lag_R.ptr, (const double *)ctx->lag_C.ptr, stacked_out, k,
                                 ctx->h, ctx->w);
}

// Gram of the cross-view block of n_img image pairs into stacked_out (fresh slots).  Always the dense kernel, also
// when the lag-structured option is on: these are the class-sum and total-sum images, a handful against the maps
// themselves, and they carry a level of (class size) x (image mean) that the raw products of the lag kernel would
// square before anything is subtracted -- the dense kernel contracts differences to the centre pixel, which do not
// see that level (measured at 30 607 images in 257 classes: C_w / C_T against the fp64 definition 1.2e-6 / 1.8e-6
// from the lag kernel, 7e-7 / 3e-7 from the dense one, and the second stage's near-degenerate filter pairs amplify
// the difference into the end-to-end histograms).
static int cross_gram(ddcca_ctx *ctx, const float *img1, const float *img2, int64_t n_img, double *stacked_out)
{
    const int k = ctx->k;
    int rc, valid = 0;
    if ((rc = launch_patch_gram(ctx, img1, img2, n_img, ctx->h, ctx->w, k, true, (double *)ctx->slots.ptr,
                                max_gram_slots(ctx, k), &valid)))
        return rc;
    return launch_gram_reduce(ctx, (const double *)ctx->slots.ptr, valid, k, stacked_out);
}

// Finish the accumulation: Gram partials -> stacked Gram, class sums -> class / total
// images -> their Grams, then the five normalised matrices in ctx->mats.
static int corr_finish(ddcca_ctx *ctx)
{
    const int k = ctx->k, D = k * k;
    const int tiles = gram_tiles(k);
    const size_t E = (size_t)tiles * 256;
    const int64_t P = (int64_t)ctx->h * ctx->w;
    const int n_cell = ctx->n_cls * ctx->G;
    int rc;
    if ((rc = ensure(ctx, ctx->stacked, 3 * E * sizeof(double)))) return rc;
    if ((rc = ensure(ctx, ctx->mats, 5 * (size_t)D * D * sizeof(double)))) return rc;
    double *st = (double *)ctx->stacked.ptr;
    if (ctx->lag_active) {
        if ((rc = lag_finish(ctx, ctx->lag_valid, ctx->lag_col_valid, st))) return rc;
    } else if ((rc = launch_gram_reduce(ctx, (const double *)ctx->slots.ptr, ctx->slots_valid, k, st))) {
        return rc;
    }

    if ((rc = ensure(ctx, ctx->class_img, 2 * (size_t)(n_cell + ctx->G) * P * sizeof(float)))) return rc;
    float *img = (float *)ctx->class_img.ptr;
    if (!ctx->class_img_ready &&
        (rc = launch_class_finalize(ctx, (const double *)ctx->class_sum.ptr, ctx->n_cls, ctx->G, P, img,
                                    ctx->cs_seg)))
        return rc;
    const size_t view_stride = (size_t)(n_cell + ctx->G) * P;
    if ((rc = cross_gram(ctx, img, img + view_stride, n_cell, st + E))) return rc;
    if ((rc = cross_gram(ctx, img + (size_t)n_cell * P, img + view_stride + (size_t)n_cell * P, ctx->G, st + 2 * E)))
        return rc;
    const double N = (double)ctx->n_maps * (double)P;
    if ((rc = launch_export(ctx, st, st + E, st + 2 * E, k, N, (double *)ctx->mats.ptr))) return rc;
    ctx->corr_exported = true;
    ctx->slots_valid = 0;
    return DDCCA_OK;
}

}  // namespace ddcca

using namespace ddcca;

extern "C" {

int ddcca_create(ddcca_ctx **out, int device, void *hip_stream)
{
    if (!out) return DDCCA_EINVAL;
    *out = nullptr;
    if (device < 0 || device >= MAX_DEVICES) return DDCCA_EINVAL;
    ddcca_ctx *ctx = new (std::nothrow) ddcca_ctx();
    if (!ctx) return DDCCA_ENOMEM;
    ctx->device = device;
    ctx->stream = (hipStream_t)hip_stream;
    *out = ctx;
    return DDCCA_OK;
}

void ddcca_destroy(ddcca_ctx *ctx)
{
    if (!ctx) return;
    bool touched = ctx->n_cu != 0;
    if (touched) {
        (void)hipSetDevice(ctx->device);
        (void)hipStreamSynchronize(ctx->stream);
        for (Buffer *b : {&ctx->lag_slots, &ctx->lag_col_slots, &ctx->lag_R, &ctx->lag_C, &ctx->prev_img, &ctx->slots, &ctx->class_sum, &ctx->class_img,
                          &ctx->stacked, &ctx->seg, &ctx->mats, &ctx->solve_ws, &ctx->flags, &ctx->maps1, &ctx->maps2, &ctx->codes, &ctx->iq_lut})
            free_buffer(*b);
        for (ProfSlot &s : ctx->prof_slot) {
            for (hipEvent_t e : s.start) (void)hipEventDestroy(e);
            for (hipEvent_t e : s.stop) (void)hipEventDestroy(e);
        }
    }
    delete ctx;
}

const char *ddcca_last_error(const ddcca_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int ddcca_status(ddcca_ctx *ctx)
{
    if (!ctx) return DDCCA_EINVAL;
    int rc;
    if ((rc = device_ready(ctx))) return rc;
    DDCCA_HIP(ctx, hipStreamSynchronize(ctx->stream));
    int host[4] = {0, 0, 0, 0};
    if (ctx->static_solve_used) {
        ctx->static_solve_used = false;
        if ((rc = static_solve_flags(ctx, host))) return rc;
    }
    if (ctx->flags.ptr) {
        int own[4] = {0, 0, 0, 0};
        DDCCA_HIP(ctx, hipMemcpy(own, ctx->flags.ptr, sizeof(own), hipMemcpyDeviceToHost));
        if (own[0] || own[1] || own[2]) DDCCA_HIP(ctx, hipMemset(ctx->flags.ptr, 0, sizeof(own)));
        for (int i = 0; i < 4; ++i) host[i] |= own[i];
    }
    if (host[0]) return fail(ctx, DDCCA_ELABEL, "class label outside [0, n_cls) seen on the device");
    if (host[1])
        return fail(ctx, DDCCA_ENUMERIC,
                    "DCCA solve: C_dd + ridge is not positive definite (NaN/Inf input or ridge too small)");
    if (host[2]) return fail(ctx, DDCCA_ENUMERIC, "DCCA solve: the Jacobi rotations did not converge");
    return DDCCA_OK;
}

int ddcca_corr_begin(ddcca_ctx *ctx, int k, int n_cls, int G, int h, int w)
{
    if (!ctx) return DDCCA_EINVAL;
    int rc;
    if ((rc = check_image_args(ctx, 0, h, w, k))) return rc;
    if (n_cls < 1 || n_cls > (1 << 20)) return fail(ctx, DDCCA_EINVAL, "n_cls must be in 1..2^20");
    if (G < 1 || G > 4096) return fail(ctx, DDCCA_EINVAL, "G (maps per sample) must be in 1..4096");
    if ((int64_t)n_cls * G > 65535) return fail(ctx, DDCCA_EINVAL, "n_cls * G must not exceed 65535");
    if ((rc = device_ready(ctx))) return rc;
    const int64_t P = (int64_t)h * w;
    const size_t E = (size_t)gram_tiles(k) * 256;
    const int max_slots = max_gram_slots(ctx, k);
    if ((rc = ensure(ctx, ctx->slots, (size_t)max_slots * E * sizeof(double)))) return rc;
    const int cs_seg = class_sum_segments((int64_t)n_cls * G, P);
    const size_t cs_bytes = (size_t)cs_seg * 2 * n_cls * G * P * sizeof(double);
    if ((rc = ensure(ctx, ctx->class_sum, cs_bytes))) return rc;
    if ((rc = launch_zero_sums(ctx, (double *)ctx->class_sum.ptr, cs_bytes / sizeof(double)))) return rc;
    if ((rc = ensure_flags(ctx))) return rc;
    ctx->lag_active = ctx->gram_arith == DDCCA_GRAM_LAG_FP32 && lag_supported(k);
    if (ctx->lag_active) {
        if ((rc = ensure(ctx, ctx->lag_slots, (size_t)max_lag_slots(ctx) * lag_slot_doubles(k) * sizeof(double))))
            return rc;
        if ((rc = ensure(ctx, ctx->lag_col_slots,
                         (size_t)max_lag_col_slots(ctx) * lag_col_slot_doubles(k) * sizeof(double))))
            return rc;
        if ((rc = ensure(ctx, ctx->lag_R, lag_slot_doubles(k) * sizeof(double)))) return rc;
        if ((rc = ensure(ctx, ctx->lag_C, lag_col_slot_doubles(k) * sizeof(double)))) return rc;
    }
    ctx->lag_valid = ctx->lag_col_valid = 0;
    ctx->k = k; ctx->n_cls = n_cls; ctx->G = G; ctx->h = h; ctx->w = w;
    ctx->cs_seg = cs_seg;
    ctx->n_maps = 0;
    ctx->slots_valid = 0;
    ctx->corr_active = true;
    ctx->corr_exported = false;
    ctx->class_img_ready = false;
    return DDCCA_OK;
}

int ddcca_corr_accumulate(ddcca_ctx *ctx, const float *v1, const float *v2, const int32_t *cls, int64_t n_img)
{
    if (!ctx) return DDCCA_EINVAL;
    if (!ctx->corr_active || ctx->corr_exported)
        return fail(ctx, DDCCA_ESTATE, "ddcca_corr_accumulate needs an open ddcca_corr_begin");
    if (n_img < 0) return fail(ctx, DDCCA_EINVAL, "negative sample count");
    if (n_img == 0) return DDCCA_OK;
    if (!v1 || !v2 || !cls) return fail(ctx, DDCCA_EINVAL, "null data pointer");
    if (n_img * (int64_t)ctx->G > (int64_t)1 << 40) return fail(ctx, DDCCA_EINVAL, "too many maps");
    int rc;
    if ((rc = device_ready(ctx))) return rc;
    const int64_t n_maps = n_img * ctx->G;
    const int64_t P = (int64_t)ctx->h * ctx->w;
    if ((rc = launch_label_check(ctx, cls, n_img, ctx->n_cls, (int *)ctx->flags.ptr))) return rc;
    if ((rc = launch_class_sum(ctx, v1, v2, cls, n_img, ctx->G, ctx->n_cls, P, (double *)ctx->class_sum.ptr,
                               ctx->cs_seg)))
        return rc;
    if ((rc = accumulate_gram(ctx, v1, v2, n_maps))) return rc;
    ctx->n_maps += n_maps;
    return DDCCA_OK;
}

int ddcca_corr_export(ddcca_ctx *ctx, double *C11, double *C22, double *C12, double *Cw, double *CT)
{
    if (!ctx) return DDCCA_EINVAL;
    if (!ctx->corr_active) return fail(ctx, DDCCA_ESTATE, "ddcca_corr_export needs ddcca_corr_begin");
    if (ctx->n_maps == 0) return fail(ctx, DDCCA_ESTATE, "nothing accumulated");
    int rc;
    if ((rc = device_ready(ctx))) return rc;
    if (!ctx->corr_exported && (rc = corr_finish(ctx))) return rc;
    const size_t bytes = (size_t)ctx->k * ctx->k * ctx->k * ctx->k * sizeof(double);
    double *dst[5] = {C11, C22, C12, Cw, CT};
    for (int i = 0; i < 5; ++i)
        if (dst[i])
            DDCCA_HIP(ctx, hipMemcpyAsync(dst[i], (const char *)ctx->mats.ptr + i * bytes, bytes,
                                          hipMemcpyDeviceToDevice, ctx->stream));
    return DDCCA_OK;
}

static int check_solve_args(ddcca_ctx *ctx, int k, int L, double ridge, const void *W1, const void *W2,
                            const void *rho)
{
    if (!valid_k(k)) return fail(ctx, DDCCA_EINVAL, "patch side k must be odd and in 3..9");
    if (L < 1 || L > k * k - 1) return fail(ctx, DDCCA_EINVAL, "L must be in 1..k*k-1");
    if (!(ridge > 0.0) || !(ridge < 1.0)) return fail(ctx, DDCCA_EINVAL, "ridge must be in (0,1)");
    if (!W1 || !W2 || !rho) return fail(ctx, DDCCA_EINVAL, "null output pointer");
    return DDCCA_OK;
}

int ddcca_solve_filters(ddcca_ctx *ctx, int L, double ridge, float *W1, float *W2, double *rho)
{
    if (!ctx) return DDCCA_EINVAL;
    if (!ctx->corr_active) return fail(ctx, DDCCA_ESTATE, "ddcca_solve_filters needs ddcca_corr_begin");
    if (ctx->n_maps == 0) return fail(ctx, DDCCA_ESTATE, "nothing accumulated");
    int rc;
    if ((rc = check_solve_args(ctx, ctx->k, L, ridge, W1, W2, rho))) return rc;
    if ((rc = device_ready(ctx))) return rc;
    if (!ctx->corr_exported && (rc = corr_finish(ctx))) return rc;
    const size_t DD = (size_t)ctx->k * ctx->k * ctx->k * ctx->k;
    const double *m = (const double *)ctx->mats.ptr;
    return launch_solve(ctx, m, m + DD, m + 3 * DD, m + 4 * DD, ctx->k, L, ridge, W1, W2, rho);
}

int ddcca_dcca_solve(ddcca_ctx *ctx, const double *C11, const double *C22, const double *Cw, const double *CT,
                     int k, int L, double ridge, float *W1, float *W2, double *rho)
{
    if (!ctx) return DDCCA_EINVAL;
    int rc;
    if ((rc = check_solve_args(ctx, k, L, ridge, W1, W2, rho))) return rc;
    if (!C11 || !C22 || !Cw || !CT) return fail(ctx, DDCCA_EINVAL, "null matrix pointer");
    if ((rc = device_ready(ctx))) return rc;
    return launch_solve(ctx, C11, C22, Cw, CT, k, L, ridge, W1, W2, rho);
}

int ddcca_dcca_solve_noalloc(ddcca_ctx *ctx, const double *C11, const double *C22, const double *Cw,
                             const double *CT, int k, int L, double ridge, float *W1, float *W2, double *rho)
{
    if (!ctx) return DDCCA_EINVAL;
    int rc;
    if ((rc = check_solve_args(ctx, k, L, ridge, W1, W2, rho))) return rc;
    if (!C11 || !C22 || !Cw || !CT) return fail(ctx, DDCCA_EINVAL, "null matrix pointer");
    if ((rc = device_ready(ctx))) return rc;
    return launch_solve_static(ctx, C11, C22, Cw, CT, k, L, ridge, W1, W2, rho);
}

int ddcca_learn_stage_filters(ddcca_ctx *ctx, const float *v1, const float *v2, const int32_t *cls, int64_t n_img,
                              int G, int h, int w, int n_cls, int k, int L, double ridge, float *W1, float *W2,
                              double *rho)
{
    if (!ctx) return DDCCA_EINVAL;
    int rc;
    if ((rc = check_image_args(ctx, n_img, h, w, k))) return rc;
    if ((rc = check_solve_args(ctx, k, L, ridge, W1, W2, rho))) return rc;
    if (n_img < 1) return fail(ctx, DDCCA_EINVAL, "need at least one sample to learn filters");
    if (!v1 || !v2 || !cls) return fail(ctx, DDCCA_EINVAL, "null data pointer");
    if ((rc = ddcca_corr_begin(ctx, k, n_cls, G, h, w))) return rc;
    if ((rc = ddcca_corr_accumulate(ctx, v1, v2, cls, n_img))) return rc;
    return ddcca_solve_filters(ctx, L, ridge, W1, W2, rho);
}

// The batch size that covers n items in the fewest batches of at most `most` items, all (nearly) equally large: a
// short last batch would run its kernels on a fraction of the chip.
static int64_t even_batch(int64_t n, int64_t most)
{
    if (n < 1) return 1;
    most = std::max<int64_t>(1, std::min(most, n));
    const int64_t batches = (n + most - 1) / most;
    return (n + batches - 1) / batches;
}

// whether the stage convolution at this patch size runs on three-piece bf16 operands
static bool conv_is_split(const ddcca_ctx *ctx, int k)
{
    return ctx->conv_arith == DDCCA_CONV_BF16X3 || (ctx->conv_arith == DDCCA_CONV_AUTO && k >= 5);
}

static int run_conv(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L, float *out)
{
    return conv_is_split(ctx, k) ? launch_conv_split(ctx, in, n, h, w, W, k, L, out)
                                 : launch_conv(ctx, in, n, h, w, W, k, L, out);
}

// The last stage fused with the output layer: no maps in memory.  In the arithmetic the convolution of this patch
// size has (so that the result is that of run_conv + launch_hash_hist bit for bit): on three-piece operands the
// convolution kernel itself hashes its maps and writes one byte per pixel and 8 filters, and the histograms are
// counted from the code maps; on the fp32 matrix instructions, the ring kernel.
static int run_conv_hash_hist(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L2,
                              int bh, int bw, int sy, int sx, void *out, int feat_type, int64_t group,
                              int64_t group_stride)
{
    if (conv_is_split(ctx, k)) {
        int rc;
        if ((rc = ensure(ctx, ctx->codes, (size_t)n * ((L2 + 7) / 8) * h * w))) return rc;
        unsigned char *codes = (unsigned char *)ctx->codes.ptr;
        if ((rc = launch_conv_split_codes(ctx, in, n, h, w, W, k, L2, codes))) return rc;
        return launch_code_hist(ctx, codes, n, L2, h, w, bh, bw, sy, sx, out, feat_type, group, group_stride);
    }
    return launch_conv_hash_hist(ctx, in, n, h, w, W, k, L2, bh, bw, sy, sx, out, feat_type, group, group_stride);
}

int ddcca_learn_next_stage_filters(ddcca_ctx *ctx, const float *v1, const float *v2, const int32_t *cls, int64_t n_img,
                                   int G_in, int h, int w, int n_cls, const float *Wp1, const float *Wp2, int k_prev,
                                   int L_prev, int k, int L, double ridge, int64_t batch_images, float *W1, float *W2,
                                   double *rho)
{
    if (!ctx) return DDCCA_EINVAL;
    int rc;
    if ((rc = check_image_args(ctx, n_img, h, w, k))) return rc;
    if ((rc = check_image_args(ctx, n_img, h, w, k_prev))) return rc;
    if ((rc = check_solve_args(ctx, k, L, ridge, W1, W2, rho))) return rc;
    if (n_img < 1) return fail(ctx, DDCCA_EINVAL, "need at least one sample to learn filters");
    if (!v1 || !v2 || !cls || !Wp1 || !Wp2) return fail(ctx, DDCCA_EINVAL, "null data pointer");
    if (G_in < 1 || L_prev < 1 || L_prev > k_prev * k_prev - 1)
        return fail(ctx, DDCCA_EINVAL, "G_in must be positive and L_prev in 1..k_prev*k_prev-1");
    if ((int64_t)G_in * L_prev > 4096) return fail(ctx, DDCCA_EINVAL, "G_in * L_prev must not exceed 4096");
    if (batch_images < 0) return fail(ctx, DDCCA_EINVAL, "negative batch size");
    const int G = G_in * L_prev;
    if ((rc = ddcca_corr_begin(ctx, k, n_cls, G, h, w))) return rc;
    const int64_t P = (int64_t)h * w;
    const int64_t cells_in = (int64_t)n_cls * G_in, n_cell = (int64_t)n_cls * G;
    // class-conditioned sum images of the next stage = previous-stage convolution of the inputs' sum images
    if ((rc = launch_label_check(ctx, cls, n_img, n_cls, (int *)ctx->flags.ptr))) return rc;
    // (their own segmentation: the sum images of the inputs are 1/L_prev of the buffer corr_begin sized)
    const int seg_in = class_sum_segments(cells_in, P);
    const size_t cs_in = (size_t)seg_in * 2 * cells_in * P * sizeof(double);
    if ((rc = ensure(ctx, ctx->class_sum, cs_in))) return rc;
    if ((rc = launch_zero_sums(ctx, (double *)ctx->class_sum.ptr, cs_in / sizeof(double)))) return rc;
    if ((rc = launch_class_sum(ctx, v1, v2, cls, n_img, G_in, n_cls, P, (double *)ctx->class_sum.ptr, seg_in)))
        return rc;
    if ((rc = ensure(ctx, ctx->prev_img, 2 * (size_t)(cells_in + G_in) * P * sizeof(float)))) return rc;
    float *pimg = (float *)ctx->prev_img.ptr;
    if ((rc = launch_class_finalize(ctx, (const double *)ctx->class_sum.ptr, n_cls, G_in, P, pimg, seg_in))) return rc;
    if ((rc = ensure(ctx, ctx->class_img, 2 * (size_t)(n_cell + G) * P * sizeof(float)))) return rc;
    float *cimg = (float *)ctx->class_img.ptr;
    if ((rc = run_conv(ctx, pimg, cells_in + G_in, h, w, Wp1, k_prev, L_prev, cimg))) return rc;
    if ((rc = run_conv(ctx, pimg + (size_t)(cells_in + G_in) * P, cells_in + G_in, h, w, Wp2, k_prev, L_prev,
                       cimg + (size_t)(n_cell + G) * P)))
        return rc;
    ctx->class_img_ready = true;
    if (ctx->next_stage_maps == DDCCA_MAPS_RECOMPUTED && !ctx->lag_active && k_prev == k) {
        // the maps never exist: the Gram kernel produces each tile of them from the input tile it holds
        if ((rc = launch_patch_gram_recomputed(ctx, v1, v2, n_img * G_in, h, w, k, Wp1, Wp2, L_prev,
                                               (double *)ctx->slots.ptr, max_gram_slots(ctx, k), &ctx->slots_valid)))
            return rc;
        ctx->n_maps += n_img * G;
        return ddcca_solve_filters(ctx, L, ridge, W1, W2, rho);
    }
    // the maps themselves, one batch of samples at a time
    const size_t per_img = (size_t)G * P * sizeof(float);
    int64_t nb = batch_images;
    if (nb == 0) nb = std::max<int64_t>(1, (int64_t)(((size_t)4 << 30) / per_img));   // 4 GiB of maps per view
    nb = std::min(nb, n_img);
    if (batch_images == 0) nb = even_batch(n_img, nb);
    if ((rc = ensure(ctx, ctx->maps1, (size_t)nb * per_img))) return rc;
    if ((rc = ensure(ctx, ctx->maps2, (size_t)nb * per_img))) return rc;
    float *m1 = (float *)ctx->maps1.ptr, *m2 = (float *)ctx->maps2.ptr;
    for (int64_t i0 = 0; i0 < n_img; i0 += nb) {
        const int64_t b = std::min(nb, n_img - i0);
        if ((rc = run_conv(ctx, v1 + (size_t)i0 * G_in * P, b * G_in, h, w, Wp1, k_prev, L_prev, m1))) return rc;
        if ((rc = run_conv(ctx, v2 + (size_t)i0 * G_in * P, b * G_in, h, w, Wp2, k_prev, L_prev, m2))) return rc;
        if ((rc = accumulate_gram(ctx, m1, m2, b * G))) return rc;
        ctx->n_maps += b * G;
    }
    return ddcca_solve_filters(ctx, L, ridge, W1, W2, rho);
}

int ddcca_set_option(ddcca_ctx *ctx, int option, int value)
{
    if (!ctx) return DDCCA_EINVAL;
    switch (option) {
        case DDCCA_OPT_CONV_ARITH:
            if (value != DDCCA_CONV_FP32 && value != DDCCA_CONV_BF16X3 && value != DDCCA_CONV_AUTO)
                return fail(ctx, DDCCA_EINVAL, "unknown convolution arithmetic");
            ctx->conv_arith = value;
            return DDCCA_OK;
        case DDCCA_OPT_GRAM_ARITH:
            if (value != DDCCA_GRAM_FP32 && value != DDCCA_GRAM_BF16X3 && value != DDCCA_GRAM_LAG_FP32)
                return fail(ctx, DDCCA_EINVAL, "unknown Gram arithmetic");
            if (ctx->corr_active && !ctx->corr_exported)
                return fail(ctx, DDCCA_ESTATE, "cannot change the Gram arithmetic during an accumulation");
            ctx->gram_arith = value;
            return DDCCA_OK;
        case DDCCA_OPT_NEXT_STAGE_MAPS:
            if (value != DDCCA_MAPS_STREAMED && value != DDCCA_MAPS_RECOMPUTED)
                return fail(ctx, DDCCA_EINVAL, "unknown next-stage map mode");
            ctx->next_stage_maps = value;
            return DDCCA_OK;
        default: return fail(ctx, DDCCA_EINVAL, "unknown option");
    }
}

int ddcca_apply_stage(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L,
                      float *out)
{
    if (!ctx) return DDCCA_EINVAL;
    int rc;
    if ((rc = check_image_args(ctx, n, h, w, k))) return rc;
    if (L < 1 || L > 64) return fail(ctx, DDCCA_EINVAL, "L must be in 1..64");
    if (n == 0) return DDCCA_OK;
    if (!in || !W || !out) return fail(ctx, DDCCA_EINVAL, "null data pointer");
    if ((rc = device_ready(ctx))) return rc;
    return run_conv(ctx, in, n, h, w, W, k, L, out);
}

static int check_hist_args(ddcca_ctx *ctx, int64_t n, int L2, int h, int w, int bh, int bw, int sy, int sx)
{
    if (n < 0) return fail(ctx, DDCCA_EINVAL, "negative map count");
    if (h < 1 || w < 1) return fail(ctx, DDCCA_EINVAL, "map height and width must be >= 1");
    if ((int64_t)h * w > (int64_t)1 << 26) return fail(ctx, DDCCA_EINVAL, "map larger than 2^26 pixels");
    if (L2 < 1 || L2 > DDCCA_MAX_L2) return fail(ctx, DDCCA_EINVAL, "L2 must be in 1..12");
    if (bh < 1 || bw < 1 || bh > h || bw > w) return fail(ctx, DDCCA_EINVAL, "block must fit inside the map");
    if (sy < 1 || sx < 1) return fail(ctx, DDCCA_EINVAL, "stride must be >= 1");
    if ((int64_t)bh * bw > 65535) return fail(ctx, DDCCA_EOVERFLOW, "block area exceeds the uint16 count range");
    return DDCCA_OK;
}

static int check_feat_type(ddcca_ctx *ctx, int feat_type)
{
    if (feat_type != DDCCA_FEAT_COUNT_U16 && feat_type != DDCCA_FEAT_IQ_F32 && feat_type != DDCCA_FEAT_IQ_F16)
        return fail(ctx, DDCCA_EINVAL, "unknown feature type");
    return DDCCA_OK;
}

static size_t feat_elem_size(int feat_type) { return feat_type == DDCCA_FEAT_IQ_F32 ? 4 : 2; }

int ddcca_hash_iq(ddcca_ctx *ctx, const float *maps, int64_t n, int L2, int h, int w, int block_h, int block_w,
                  int stride_y, int stride_x, int feat_type, void *out)
{
    if (!ctx) return DDCCA_EINVAL;
    int rc;
    if ((rc = check_feat_type(ctx, feat_type))) return rc;
    if ((rc = check_hist_args(ctx, n, L2, h, w, block_h, block_w, stride_y, stride_x))) return rc;
    if (n == 0) return DDCCA_OK;
    if (!maps || !out) return fail(ctx, DDCCA_EINVAL, "null data pointer");
    if ((rc = device_ready(ctx))) return rc;
    const int64_t A = (int64_t)((h - block_h) / stride_y + 1) * ((w - block_w) / stride_x + 1);
    return launch_hash_hist(ctx, maps, n, L2, h, w, block_h, block_w, stride_y, stride_x, out, feat_type, 1,
                            A * ((int64_t)1 << L2));
}

int ddcca_hash_histogram(ddcca_ctx *ctx, const float *maps, int64_t n, int L2, int h, int w, int block_h,
                         int block_w, int stride_y, int stride_x, uint16_t *hist)
{
    return ddcca_hash_iq(ctx, maps, n, L2, h, w, block_h, block_w, stride_y, stride_x, DDCCA_FEAT_COUNT_U16, hist);
}

int ddcca_extract_features(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t m, int h, int w,
                           const ddcca_model *model, uint16_t *feat)
{
    return ddcca_extract_iq_features(ctx, v1, v2, m, h, w, model, DDCCA_FEAT_COUNT_U16, feat);
}

static int extract_impl(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t m, int h, int w,
                        const ddcca_model *model, int feat_type, void *feat, bool fused)
{
    if (!ctx) return DDCCA_EINVAL;
    if (!model) return fail(ctx, DDCCA_EINVAL, "null model");
    int rc;
    if ((rc = check_feat_type(ctx, feat_type))) return rc;
    if ((rc = check_image_args(ctx, m, h, w, model->k))) return rc;
    if (model->L1 < 1 || model->L1 > 64) return fail(ctx, DDCCA_EINVAL, "L1 must be in 1..64");
    if ((rc = check_hist_args(ctx, m, model->L2, h, w, model->block_h, model->block_w, model->stride_y,
                              model->stride_x)))
        return rc;
    if (model->batch_images < 0) return fail(ctx, DDCCA_EINVAL, "negative batch size");
    for (int s = 0; s < 2; ++s)
        for (int d = 0; d < 2; ++d)
            if (!model->W[s][d]) return fail(ctx, DDCCA_EINVAL, "null filter pointer in model");
    if (m == 0) return DDCCA_OK;
    if (!v1 || !v2 || !feat) return fail(ctx, DDCCA_EINVAL, "null data pointer");
    if ((rc = device_ready(ctx))) return rc;

    const int L1 = model->L1, L2 = model->L2, k = model->k;
    const int64_t P = (int64_t)h * w;
    const int64_t A = (int64_t)((h - model->block_h) / model->stride_y + 1) *
                      ((w - model->block_w) / model->stride_x + 1);
    const int64_t bins = (int64_t)1 << L2;
    // default batch: the largest map buffer of one view for one batch (stage-2 maps; stage-1 maps when the
    // second stage is fused with the output layer) takes about 4 GiB
    int64_t batch = model->batch_images;
    if (batch == 0) {
        const double per_image = (double)L1 * (fused ? 1 : L2) * P * sizeof(float);
        batch = even_batch(m, (int64_t)std::max(1.0, 4.0 * 1073741824.0 / per_image));
    }
    batch = std::min(batch, m);
    if ((rc = ensure(ctx, ctx->maps1, (size_t)batch * L1 * P * sizeof(float)))) return rc;
    if (!fused && (rc = ensure(ctx, ctx->maps2, (size_t)batch * L1 * L2 * P * sizeof(float)))) return rc;
    float *y = (float *)ctx->maps1.ptr, *z = (float *)ctx->maps2.ptr;
    const float *views[2] = {v1, v2};
    for (int64_t m0 = 0; m0 < m; m0 += batch) {
        const int64_t mb = std::min(batch, m - m0);
        for (int d = 0; d < 2; ++d) {
            if ((rc = run_conv(ctx, views[d] + m0 * P, mb, h, w, model->W[0][d], k, L1, y))) return rc;
            if (!fused && (rc = run_conv(ctx, y, mb * L1, h, w, model->W[1][d], k, L2, z))) return rc;
            void *dst = reinterpret_cast<char *>(feat) + ((m0 * 2 + d) * L1) * A * bins * feat_elem_size(feat_type);
            if (fused)
                rc = run_conv_hash_hist(ctx, y, mb * L1, h, w, model->W[1][d], k, L2, model->block_h,
                                        model->block_w, model->stride_y, model->stride_x, dst, feat_type, L1,
                                        2 * L1 * A * bins);
            else
                rc = launch_hash_hist(ctx, z, mb * L1, L2, h, w, model->block_h, model->block_w, model->stride_y,
                                      model->stride_x, dst, feat_type, L1, 2 * L1 * A * bins);
            if (rc) return rc;
        }
    }
    return DDCCA_OK;
}

int ddcca_extract_iq_features(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t m, int h, int w,
                              const ddcca_model *model, int feat_type, void *feat)
{
    return extract_impl(ctx, v1, v2, m, h, w, model, feat_type, feat, false);
}

int ddcca_extract_features_fused(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t m, int h, int w,
                                 const ddcca_model *model, int feat_type, void *feat)
{
    return extract_impl(ctx, v1, v2, m, h, w, model, feat_type, feat, true);
}

int ddcca_apply_stage_hash(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L2,
                           int block_h, int block_w, int stride_y, int stride_x, int feat_type, void *out)
{
    if (!ctx) return DDCCA_EINVAL;
    int rc;
    if ((rc = check_feat_type(ctx, feat_type))) return rc;
    if ((rc = check_image_args(ctx, n, h, w, k))) return rc;
    if ((rc = check_hist_args(ctx, n, L2, h, w, block_h, block_w, stride_y, stride_x))) return rc;
    if (n == 0) return DDCCA_OK;
    if (!in || !W || !out) return fail(ctx, DDCCA_EINVAL, "null data pointer");
    if ((rc = device_ready(ctx))) return rc;
    const int64_t A = (int64_t)((h - block_h) / stride_y + 1) * ((w - block_w) / stride_x + 1);
    return run_conv_hash_hist(ctx, in, n, h, w, W, k, L2, block_h, block_w, stride_y, stride_x, out, feat_type, 1,
                              A * ((int64_t)1 << L2));
}

int ddcca_profile_enable(ddcca_ctx *ctx, int on)
{
    if (!ctx) return DDCCA_EINVAL;
    ctx->prof = on != 0;
    return DDCCA_OK;
}

int ddcca_profile_select(ddcca_ctx *ctx, unsigned int kernel_mask)
{
    if (!ctx) return DDCCA_EINVAL;
    if (!(kernel_mask & ((1u << DDCCA_K_COUNT) - 1u))) return fail(ctx, DDCCA_EINVAL, "profile mask selects no kernel");
    ctx->prof_mask = kernel_mask;
    return DDCCA_OK;
}

int ddcca_profile_reset(ddcca_ctx *ctx)
{
    if (!ctx) return DDCCA_EINVAL;
    if (ctx->n_cu) DDCCA_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (ProfSlot &s : ctx->prof_slot) {
        s.used = 0;
        s.carried_ms = 0.0;
        s.launches = 0;
    }
    return DDCCA_OK;
}

int ddcca_profile_read(ddcca_ctx *ctx, int kernel_id, double *total_ms, int64_t *launches)
{
    if (!ctx) return DDCCA_EINVAL;
    if (kernel_id < 0 || kernel_id >= DDCCA_K_COUNT || !total_ms || !launches)
        return fail(ctx, DDCCA_EINVAL, "bad kernel id or null output");
    ProfSlot &s = ctx->prof_slot[kernel_id];
    double ms = s.carried_ms;
    if (s.used) {
        int rc;
        if ((rc = device_ready(ctx))) return rc;
        DDCCA_HIP(ctx, hipStreamSynchronize(ctx->stream));
        for (size_t i = 0; i < s.used; ++i) {
            float t = 0.f;
            DDCCA_HIP(ctx, hipEventElapsedTime(&t, s.start[i], s.stop[i]));
            ms += t;
        }
    }
    *total_ms = ms;
    *launches = s.launches;
    return DDCCA_OK;
}

}  // extern "C"
