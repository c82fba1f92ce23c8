/*
 * ddcca.h -- C ABI of the MI355X (gfx950) two-stage DDCCANet feature-extractor hot path.
 *
 * The calls follow the paper's statement of the problem: two aligned views of M images
 * (M x p x q tensors, Section II-A) plus class labels go in; per stage the DDCCA filters
 * W^1, W^2 come out (Eq. 2-5), every image is convolved with them (Eq. 6), and the
 * output layer hashes the last stage's maps into per-block code histograms (Eq. 7-9,
 * Section II-C, Eq. 11-12).
 *
 * General rules
 *   - Every data pointer is a DEVICE pointer owned by the caller (for example the
 *     data_ptr() of a PyTorch tensor on the context's GPU).  Host pointers are not
 *     accepted.  The library reads/writes them only inside the call's enqueued work and
 *     keeps no reference afterwards.
 *   - All calls enqueue on the context's stream and return without synchronising,
 *     unless stated otherwise.  Scratch memory is owned by the context, grown on
 *     demand (hipMalloc) and released by ddcca_destroy.
 *   - Layouts are dense row-major, innermost index x.  Images: [n][h][w] float.
 *     A patch / filter element is a = dy*k + dx (Eq. 4-5 read row-major).
 *     Patches are taken at every pixel with zero padding r=(k-1)/2 (Eq. 1 has M*p*q
 *     columns) and each patch has its own mean removed.
 *   - Return value: DDCCA_OK (0) or a negative DDCCA_E* code.  Arguments are validated
 *     on the host before anything is launched; no C++ exception crosses the boundary.
 *     ddcca_last_error() gives a text for the last failure on that context.
 *   - A context is not thread-safe; calls on one context must not overlap.
 */
#ifndef DDCCA_H
#define DDCCA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DDCCA_OK          0
#define DDCCA_EINVAL    (-1)   /* null pointer, k even or outside 3..9, L outside 1..k*k-1, L2 > 12, block > image, stride < 1, n < 0 */
#define DDCCA_ESTATE    (-2)   /* call order: accumulate/export/solve without a matching ddcca_corr_begin */
#define DDCCA_ENOMEM    (-3)   /* scratch allocation failed */
#define DDCCA_EHIP      (-4)   /* HIP runtime error (no GPU, launch failure, ...) */
#define DDCCA_EOVERFLOW (-5)   /* a histogram count would not fit uint16 (block area > 65535) */
#define DDCCA_ELABEL    (-6)   /* a class label outside [0, n_cls) was seen on the device */
#define DDCCA_ENUMERIC  (-7)   /* the DCCA solve broke down on the device: C_dd + ridge not positive definite
                                  (NaN/Inf in the matrices, ridge too small), or no convergence */

#define DDCCA_MIN_K   3
#define DDCCA_MAX_K   9
#define DDCCA_MAX_L2 12

typedef struct ddcca_ctx ddcca_ctx;

/* Create a context bound to GPU `device` and to `hip_stream` (a hipStream_t, borrowed;
 * NULL = the device's default stream).  Touches no GPU state by itself, so it succeeds
 * on a machine without a GPU; the first call that needs the GPU then fails with
 * DDCCA_EHIP. */
int ddcca_create(ddcca_ctx **out, int device, void *hip_stream);
void ddcca_destroy(ddcca_ctx *ctx);
const char *ddcca_last_error(const ddcca_ctx *ctx);

/* Synchronise the context's stream and report sticky device-side conditions
 * (DDCCA_ELABEL, DDCCA_ENUMERIC; the condition is cleared by the call that reports it)
 * or a pending HIP error.  The calls above the device cannot see these conditions when
 * they return (nothing synchronises), so: samples with a bad label are left out of C_w
 * and C_T, and every solve that runs while that condition is pending writes NaN filters
 * and NaN rho instead of filters of inconsistent matrices; a solve that breaks down
 * leaves whatever its arithmetic produced (NaN for a non-positive pivot).  A caller that
 * replays captured work calls ddcca_status after the replay. */
int ddcca_status(ddcca_ctx *ctx);

/* ---- correlation accumulation, streamed over batches (Section III, Eq. 13-15) -------
 * begin -> accumulate(batch)* -> export / solve.
 * A batch is n_img samples of G maps each: v1, v2 are [n_img][G][h][w]; map g of view 1
 * pairs with map g of view 2 (stage 1: G = 1; stage 2: G = L1 and the maps are the
 * stage-1 outputs).  cls is [n_img] int32 on the device, values in [0, n_cls).
 * Accumulated: the sums over all patches of x1 x1^T, x2 x2^T, x1 x2^T, and per
 * (class, g) cell the pixel-wise sums of the member maps, from which the same-class
 * pair sum C_w and the all-pairs sum C_T follow (Section II-A: C~ = C_w - C_b,
 * C_b = C_T - C_w).  The split of the samples into batches changes the result only
 * through the order of the fp32 partial sums inside a batch (relative 1e-6 or less); for
 * a given split the result is reproducible bit for bit. */
int ddcca_corr_begin(ddcca_ctx *ctx, int k, int n_cls, int G, int h, int w);
int ddcca_corr_accumulate(ddcca_ctx *ctx, const float *v1, const float *v2, const int32_t *cls,
                          int64_t n_img);
/* Write the matrices, each divided by the number of patches N = (#maps)*h*w, as
 * [k*k][k*k] doubles.  Any pointer may be NULL.  May be called once per begin. */
int ddcca_corr_export(ddcca_ctx *ctx, double *C11, double *C22, double *C12, double *Cw,
                      double *CT);
/* Solve Eq. 2-3 on the accumulated matrices (runs the export step itself if it has not
 * run yet): see ddcca_dcca_solve for the outputs. */
int ddcca_solve_filters(ddcca_ctx *ctx, int L, double ridge, float *W1, float *W2, double *rho);

/* Eq. 2-3 for given matrices (all [D][D] doubles, D = k*k):
 *   maximise w1^T C~ w2,  C~ = 2 C_w - C_T,  subject to w_d^T B_d w_d = 1,
 *   B_d = C_dd + ridge * trace(C_dd)/D * I   (C_dd alone is singular after mean removal).
 * Returns the L leading pairs in descending rho, pairs mutually B-orthogonal, the sign
 * of each pair fixed so that the largest-magnitude entry of w1 is positive (lowest
 * index on ties; w2 flips with it).  W1, W2: [L][k][k] float; rho: [L] double. */
int ddcca_dcca_solve(ddcca_ctx *ctx, const double *C11, const double *C22, const double *Cw,
                     const double *CT, int k, int L, double ridge, float *W1, float *W2,
                     double *rho);

/* ddcca_dcca_solve for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernel, same results bit for bit; the call makes no hipMalloc / hipFree and records no
 * timing events (ddcca_profile_* does not see it).  The kernel's scratch -- two D x D
 * double matrices and the int[4] of sticky conditions -- is a file-scope device array of
 * 104 992 bytes sized for k = 9, the largest k of the library (a larger k is DDCCA_EINVAL
 * like everywhere else); each GPU the library runs on holds its copy until the process
 * ends.  All contexts and calls on one GPU share that array: calls of this function that
 * overlap on one GPU (different streams or threads) race; calls on one stream are
 * ordered and safe.  Nothing in it needs to start at zero except the condition flags,
 * which are zero when the library is loaded and are cleared by the ddcca_status call that
 * reports them -- on the context that made the call, for the whole GPU. */
int ddcca_dcca_solve_noalloc(ddcca_ctx *ctx, const double *C11, const double *C22,
                             const double *Cw, const double *CT, int k, int L, double ridge,
                             float *W1, float *W2, double *rho);

/* ---- the four calls of the path ----------------------------------------------------- */

/* Learn one stage's filters from all samples at once (Section II-A; begin +
 * accumulate + solve). */
int ddcca_learn_stage_filters(ddcca_ctx *ctx, const float *v1, const float *v2, const int32_t *cls,
                              int64_t n_img, int G, int h, int w, int n_cls, int k, int L,
                              double ridge, float *W1, float *W2, double *rho);

/* Eq. 6: out[n][g][y][x] = sum_{dy,dx} W[g][dy][dx] * in_pad[n][y+dy-r][x+dx-r]
 * (cross-correlation, zero padding).  in: [n][h][w]; W: [L][k][k]; out: [n][L][h][w]. */
int ddcca_apply_stage(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W,
                      int k, int L, float *out);

/* Eq. 7-9 + Section II-C: code = sum_l 2^(l-1) [maps[n][l-1][y][x] > 0]; the code map is
 * cut into block_h x block_w blocks with top-left corners (i*stride_y, j*stride_x), all
 * blocks fully inside the map; hist[n][i][j][t] counts code t in block (i,j).
 * maps: [n][L2][h][w] float; hist: [n][nby][nbx][1<<L2] uint16,
 * nby = (h-block_h)/stride_y + 1, nbx = (w-block_w)/stride_x + 1. */
int ddcca_hash_histogram(ddcca_ctx *ctx, const float *maps, int64_t n, int L2, int h, int w,
                         int block_h, int block_w, int stride_y, int stride_x, uint16_t *hist);

typedef struct ddcca_model {
    int k, L1, L2;
    int block_h, block_w, stride_y, stride_x;
    const float *W[2][2];     /* W[stage][view]: device, [L_stage][k][k] */
    int64_t batch_images;     /* images per internal batch; 0 = equal batches whose maps take at most 4 GiB per view */
} ddcca_model;

/* Both stages and the output layer for m new image pairs with a learned model:
 * feat[m][view][g][i][j][t], g < L1 (Eq. 11-12: per view the L1 block-histogram sets,
 * views concatenated per image).  Stage-2 maps are produced batch by batch in context
 * scratch and never leave the GPU. */
int ddcca_extract_features(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t m, int h,
                           int w, const ddcca_model *model, uint16_t *feat);

/* ---- information-quality form of the output layer (Eq. 10-12) -------------------------
 * Eq. 10 turns the code distribution p(t) of every block into o = -log p(t) (natural
 * logarithm).  p(t) is taken with one pseudo-count per bin,
 *     p(t) = (count(t) + 1) / (block_h*block_w + 2^L2),
 * so that a code absent from a block (where Eq. 10 is undefined) gets the finite value
 * log(block_h*block_w + 2^L2) and the p(t) of a block still sum to one.
 * feat_type selects the element type of the output: DDCCA_FEAT_IQ_F32 (float) or
 * DDCCA_FEAT_IQ_F16 (IEEE half, the fp32 value rounded to nearest); DDCCA_FEAT_COUNT_U16
 * gives the raw counts (the same as the calls above).  Layouts are those of
 * ddcca_hash_histogram / ddcca_extract_features with the element type replaced.
 * fp32 values are within one unit in the last place of the exactly rounded result. */
#define DDCCA_FEAT_COUNT_U16 0
#define DDCCA_FEAT_IQ_F32    1
#define DDCCA_FEAT_IQ_F16    2
int ddcca_hash_iq(ddcca_ctx *ctx, const float *maps, int64_t n, int L2, int h, int w, int block_h,
                  int block_w, int stride_y, int stride_x, int feat_type, void *out);
int ddcca_extract_iq_features(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t m, int h,
                              int w, const ddcca_model *model, int feat_type, void *feat);

/* ---- fused last stage ------------------------------------------------------------------
 * Eq. 6 with the L2 filters W followed by the output layer (Eq. 7-12) without the maps in
 * memory: the L2 maps of every input map are hashed as they are computed and never written.
 * The convolution runs in the arithmetic DDCCA_OPT_CONV_ARITH gives this patch size, in the
 * same order as ddcca_apply_stage, so the result is that of ddcca_apply_stage followed by
 * ddcca_hash_iq on the same context, bit for bit.  With the fp32 matrix instructions it is
 * one kernel (convolution, hashing and histograms around a ring of block rows in LDS); with
 * three-piece bf16 operands the convolution kernel writes the hash codes of its maps (one
 * byte per pixel and 8 filters, context scratch) and a second kernel counts the histograms
 * from those.  in: [n][h][w]; W: [L2][k][k]; out as ddcca_hash_iq. */
int ddcca_apply_stage_hash(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W,
                           int k, int L2, int block_h, int block_w, int stride_y, int stride_x,
                           int feat_type, void *out);
/* ddcca_extract_iq_features with the second stage and the output layer fused: the same
 * output, bit for bit; only the stage-1 maps of a batch (and, with three-piece operands,
 * its hash codes) are held in context scratch. */
int ddcca_extract_features_fused(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t m, int h,
                                 int w, const ddcca_model *model, int feat_type, void *feat);

/* ---- options ---------------------------------------------------------------------------
 * DDCCA_OPT_CONV_ARITH selects the arithmetic of the stage convolution (Eq. 6) in
 * ddcca_apply_stage, ddcca_learn_next_stage_filters and both stages of
 * ddcca_extract_features / ddcca_extract_iq_features and their fused forms:
 *   DDCCA_CONV_FP32   fp32 products and sums on the fp32 matrix instructions;
 *   DDCCA_CONV_BF16X3 every fp32 operand split exactly into three bf16 pieces and the six
 *                     significant piece products summed in fp32 on the bf16 matrix pipeline:
 *                     the accuracy of an fp32 dot product (the dropped products are below
 *                     2^-24 relative), another rounding order, several times the matrix rate;
 *   DDCCA_CONV_AUTO   (default) the faster of the two for the patch size: DDCCA_CONV_BF16X3
 *                     from k = 5 on (there the fp32 matrix instructions, not the memory,
 *                     bound the fp32 kernel), DDCCA_CONV_FP32 at k = 3.
 * DDCCA_OPT_GRAM_ARITH selects the arithmetic of the patch-Gram accumulation (Section II-A
 * matrices) in the same way: DDCCA_GRAM_FP32 (default) or DDCCA_GRAM_BF16X3.  Accumulation
 * across tiles stays fp64 in either.
 *   DDCCA_GRAM_LAG_FP32   the same matrices from the lag structure of the patch Gram: with the
 *                     images extended by zeros, the raw Gram entry of taps a and b summed over
 *                     all patch centres of the plane is the correlation of the two views at
 *                     lag s_b - s_a, (2k-1)^2 values per view pair instead of k^4, computed on
 *                     the fp32 matrix instructions and added up in fp64 row by row; the terms
 *                     of the first and last (k-1)/2 image rows and columns, which the centres
 *                     outside the image contribute, are kept apart and taken out exactly.
 *                     Same result up to fp32 rounding (same bars), several times fewer matrix
 *                     instructions.  k = 9 has 17 lags per axis against the 16 rows of the
 *                     matrix instruction: it keeps the lags -8 .. 7 for the four ordered view
 *                     pairs, reads a lag with a component +8 as the exchanged pair at the
 *                     negated lag, and sums the one remaining tap pair (opposite patch
 *                     corners) directly.
 * DDCCA_OPT_NEXT_STAGE_MAPS selects where ddcca_learn_next_stage_filters gets the maps of the
 * previous stage from (Section II-B on Section II-A):
 *   DDCCA_MAPS_STREAMED   (default) convolved batch by batch into a scratch buffer and read
 *                     back by the Gram accumulation;
 *   DDCCA_MAPS_RECOMPUTED the Gram kernel holds the INPUT tile (with the halo of both stages) in
 *                     LDS and forms each map tile from it as it needs it (fp32 fused
 *                     multiply-adds in tap order): the maps never exist in memory.  Same
 *                     matrices up to the rounding order of the convolution (same bars).  Used
 *                     when k_prev == k and the Gram arithmetic is not DDCCA_GRAM_LAG_FP32;
 *                     otherwise the call proceeds as with DDCCA_MAPS_STREAMED.  The Gram is
 *                     bound by the matrix unit, where the recomputation is paid in full,
 *                     while the convolution it replaces is bound by memory: this mode trades
 *                     time for memory traffic and scratch space.
 * Returns DDCCA_EINVAL for an unknown option or value, DDCCA_ESTATE when the Gram
 * arithmetic is changed between ddcca_corr_begin and the export / solve of that
 * accumulation. */
#define DDCCA_OPT_CONV_ARITH 1
#define DDCCA_CONV_FP32      0
#define DDCCA_CONV_BF16X3    1
#define DDCCA_CONV_AUTO      2
#define DDCCA_OPT_GRAM_ARITH 2
#define DDCCA_GRAM_FP32      0
#define DDCCA_GRAM_BF16X3    1
#define DDCCA_GRAM_LAG_FP32  2
#define DDCCA_OPT_NEXT_STAGE_MAPS 3
#define DDCCA_MAPS_STREAMED   0
#define DDCCA_MAPS_RECOMPUTED 1
int ddcca_set_option(ddcca_ctx *ctx, int option, int value);

/* Learn the filters of the stage that follows a given stage (Section II-B: the second stage
 * is learned on the maps of the first; Section II-A for the matrices) without holding those
 * maps: the result of ddcca_apply_stage(v_d, Wp_d) for both views followed by
 * ddcca_learn_stage_filters on the maps with G = G_in * L_prev.
 *   v1, v2 : DEVICE, [n_img][G_in][h][w] float, the INPUTS of the previous stage
 *   Wp1, Wp2 : DEVICE, [L_prev][k_prev][k_prev] float, the previous stage's filters per view
 *   batch_images : samples whose maps exist at a time (0 = equal batches of at most 4 GiB per view);
 *                  it changes the result only through the order of the fp32 partial sums
 *                  inside a batch (relative 1e-6 or less)
 * Every batch is convolved into a scratch buffer of the context and accumulated at once.
 * The class-conditioned sum images (the C_w and C_T terms) are formed as the previous-stage
 * convolution of the inputs' sum images -- the convolution of Eq. 6 is linear -- so they
 * differ from the sums of the fp32 maps by fp32 rounding only (relative 1e-7 per pixel).
 * The convolution arithmetic follows DDCCA_OPT_CONV_ARITH.  Other arguments, outputs and
 * errors as in ddcca_learn_stage_filters; additionally DDCCA_EINVAL when L_prev is outside
 * 1..k_prev*k_prev-1, G_in * L_prev exceeds 4096 or batch_images is negative. */
int ddcca_learn_next_stage_filters(ddcca_ctx *ctx, const float *v1, const float *v2,
                                   const int32_t *cls, int64_t n_img, int G_in, int h, int w,
                                   int n_cls, const float *Wp1, const float *Wp2, int k_prev,
                                   int L_prev, int k, int L, double ridge, int64_t batch_images,
                                   float *W1, float *W2, double *rho);

/* ---- per-kernel timing (HIP events on the context's stream) -------------------------- */
enum {
    DDCCA_K_GRAM = 0,     /* patch-Gram accumulation over the input maps (all tiles) */
    DDCCA_K_CLASS_SUM,    /* per-(class,g) image sums */
    DDCCA_K_REDUCE,       /* cross-workgroup reduction / export of the matrices */
    DDCCA_K_SOLVE,        /* DCCA solve */
    DDCCA_K_CONV,         /* stage convolution */
    DDCCA_K_HASH_HIST,    /* hashing + block histogram */
    DDCCA_K_GRAM_CROSS,   /* patch-Gram of the class-sum / total-sum images (cross-view tiles only) */
    DDCCA_K_CONV_HASH_HIST, /* last stage convolution fused with hashing + block histogram */
    DDCCA_K_COUNT
};
/* While enabled, every kernel launch is bracketed by a pair of events. */
int ddcca_profile_enable(ddcca_ctx *ctx, int on);
/* Restrict the bracketing to the kernel ids whose bit is set (bit i = id i; default and ~0u: all).  A pair of
 * events costs a few microseconds of stream time per launch, which a whole-path measurement that needs one
 * kernel's durations need not pay for the others.  DDCCA_EINVAL for a mask without any known id. */
int ddcca_profile_select(ddcca_ctx *ctx, unsigned int kernel_mask);
/* Synchronises the stream; total_ms / launches since the last reset for one kernel id. */
int ddcca_profile_read(ddcca_ctx *ctx, int kernel_id, double *total_ms, int64_t *launches);
int ddcca_profile_reset(ddcca_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* DDCCA_H */
