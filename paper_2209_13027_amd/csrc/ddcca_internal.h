// Internal declarations shared by the HIP translation units of libddcca.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <string>
#include <vector>

#include "../../include/ddcca.h"

namespace ddcca {

// A grow-on-demand device buffer owned by the context.
struct Buffer {
    void *ptr = nullptr;
    size_t bytes = 0;
};

struct ProfSlot {
    std::vector<hipEvent_t> start, stop;   // pairs recorded since the last reset
    size_t used = 0;
    double carried_ms = 0.0;               // time folded in from recycled pairs
    int64_t launches = 0;
};

}  // namespace ddcca

struct ddcca_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    std::string err;
    int n_cu = 0;                           // compute units of the device (lazy)

    // ---- correlation accumulation state (between corr_begin and export/solve)
    bool corr_active = false;
    bool corr_exported = false;
    int k = 0, n_cls = 0, G = 0, h = 0, w = 0;
    int64_t n_maps = 0;                     // maps accumulated so far (per view)
    int slots_valid = 0;                    // Gram partial slots holding data
    ddcca::Buffer slots;                    // [max_slots][tiles*256] double
    ddcca::Buffer class_sum;                // [cs_seg][2][n_cls*G][h*w] double
    int cs_seg = 1;                         // sample segments of the class-sum pass
    ddcca::Buffer class_img;                // [2][n_cls*G + G][h*w] float
    bool class_img_ready = false;           // class_img was filled directly (not from class_sum)
    ddcca::Buffer prev_img;                 // sum images of the previous stage's inputs (next-stage learning)
    ddcca::Buffer stacked;                  // 3 x [tiles*256] double (main, class, total)
    bool lag_active = false;                // this accumulation runs lag-structured (option set)
    int lag_valid = 0, lag_col_valid = 0;   // lag slots holding data
    ddcca::Buffer lag_slots, lag_col_slots; // per-workgroup lag statistics (rows / border columns)
    ddcca::Buffer lag_R, lag_C;             // the same, reduced
    ddcca::Buffer seg;                      // reduction segments
    ddcca::Buffer mats;                     // 5 x [D][D] double: C11 C22 C12 Cw CT
    ddcca::Buffer solve_ws;                 // solver scratch (global part)
    ddcca::Buffer flags;                    // int[4]: [0] label error, [1] Cholesky pivot, [2] Jacobi sweeps exhausted
    bool static_solve_used = false;         // ddcca_dcca_solve_noalloc ran: its conditions sit in the static scratch
    ddcca::Buffer maps1, maps2;             // extract_features scratch
    ddcca::Buffer codes;                    // hash codes of a batch, one byte per pixel (fused last stage)
    ddcca::Buffer iq_lut;                   // information-quality table of the output layer
    int64_t iq_lut_total = 0;               // block area + bins the table was built for (0 = none)
    int iq_lut_n = 0;

    int conv_arith = DDCCA_CONV_AUTO;       // DDCCA_OPT_CONV_ARITH
    int gram_arith = DDCCA_GRAM_FP32;       // DDCCA_OPT_GRAM_ARITH
    int next_stage_maps = DDCCA_MAPS_STREAMED;   // DDCCA_OPT_NEXT_STAGE_MAPS

    // ---- profiling
    bool prof = false;
    unsigned prof_mask = ~0u;               // kernel ids that are timed while prof is on
    ddcca::ProfSlot prof_slot[DDCCA_K_COUNT];
};

namespace ddcca {

int fail(ddcca_ctx *ctx, int code, const std::string &msg);
int hip_fail(ddcca_ctx *ctx, hipError_t e, const char *what);
int ensure(ddcca_ctx *ctx, Buffer &b, size_t bytes);     // grow; contents undefined after growth
int device_ready(ddcca_ctx *ctx);                        // set device, query CU count
int ensure_flags(ddcca_ctx *ctx);                        // the device int[4] of sticky conditions, zeroed once
constexpr int MAX_DEVICES = 64;                          // per-device host tables (kernel attributes) are this long

#define DDCCA_HIP(ctx, call)                                         \
    do {                                                             \
        hipError_t e__ = (call);                                     \
        if (e__ != hipSuccess) return ddcca::hip_fail(ctx, e__, #call); \
    } while (0)

// RAII bracket: records an event pair around a launch when profiling is on.
struct ProfScope {
    ddcca_ctx *ctx;
    int id;
    ProfScope(ddcca_ctx *c, int kernel_id);
    ~ProfScope();
};

// ---- geometry of the stacked (two views) patch Gram --------------------------------
// The stacked vector z = [y1; y2] (patches minus their centre pixel, centre entry dropped)
// has 2(D-1) entries, D = k*k.  Its Gram is computed in 16x16 tiles, upper block-triangle
// only; tile (bi,bj), bi <= bj, is number bi*NB - bi(bi-1)/2 + bj - bi.  Inside a slot, tile t /
// accumulator register v / lane l sits at (t*4 + v)*64 + l and holds Gram entry
// (16*bi + 4*(l/16) + v, 16*bj + l%16).
inline int gram_blocks(int k) { return (2 * (k * k - 1)) / 16; }
inline int gram_tiles(int k) { int nb = gram_blocks(k); return nb * (nb + 1) / 2; }

// ---- kernel launchers (each validates nothing; callers have validated) --------------
// cross_only: accumulate only the view-1 x view-2 block (the other tiles of the slots are
// then undefined and must not be read).
int launch_patch_gram(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t n_maps, int h, int w,
                      int k, bool cross_only, double *slots, int max_slots, int *slots_valid);
// the same over the maps W_l * input (previous stage, same patch size), recomputed tile by tile inside the kernel
int launch_patch_gram_recomputed(ddcca_ctx *ctx, const float *in1, const float *in2, int64_t n_inputs, int h, int w,
                                 int k, const float *Wp1, const float *Wp2, int L_prev, double *slots, int max_slots,
                                 int *slots_valid);
int max_gram_slots(ddcca_ctx *ctx, int k);
int launch_gram_reduce(ddcca_ctx *ctx, const double *slots, int n_slots, int k, double *stacked);
// the same fixed-order sum for slots of E doubles each
int launch_reduce_slots(ddcca_ctx *ctx, const double *slots, int n_slots, int E, double *out);

// ---- lag-structured accumulation (DDCCA_GRAM_LAG_FP32) ----------------------------------------
bool lag_supported(int k);
int max_lag_slots(ddcca_ctx *ctx);
int max_lag_col_slots(ddcca_ctx *ctx);
size_t lag_slot_doubles(int k);       // lag correlations: all rows + the r top and r bottom rows, per pair type
size_t lag_col_slot_doubles(int k);   // border columns and corners
// adds the lag statistics of n_maps map pairs to the two slot sets
int launch_lag_gram(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t n_maps, int h, int w, int k,
                    double *slots, int max_slots, int *slots_valid, double *col_slots, int max_col_slots,
                    int *col_slots_valid);
// stacked <- Gram of y = x - x_centre over the patches of the image, from the reduced statistics R (rows) and C
// (columns), in the layout of the dense kernel's reduced slots
int launch_lag_to_stacked(ddcca_ctx *ctx, const double *R, const double *C, double *stacked, int k, int h, int w);
int launch_export(ddcca_ctx *ctx, const double *stacked_main, const double *stacked_cls,
                  const double *stacked_tot, int k, double n_patches, double *mats);
int launch_label_check(ddcca_ctx *ctx, const int32_t *cls, int64_t n_img, int n_cls, int *flag);
int class_sum_segments(int64_t n_cell, int64_t P);        // sample segments that fill the chip
int launch_zero_sums(ddcca_ctx *ctx, double *sums, size_t n /* doubles, even */);
int launch_class_sum(ddcca_ctx *ctx, const float *v1, const float *v2, const int32_t *cls, int64_t n_img,
                     int G, int n_cls, int64_t P, double *sums /* [n_seg][2][n_cls*G][P] */, int n_seg);
int launch_class_finalize(ddcca_ctx *ctx, const double *sums, int n_cls, int G, int64_t P,
                          float *img /* [2][n_cls*G + G][P] */, int n_seg);
int launch_solve(ddcca_ctx *ctx, const double *C11, const double *C22, const double *Cw, const double *CT,
                 int k, int L, double ridge, float *W1, float *W2, double *rho);
// the same solve with its scratch in a file-scope device array (no allocation, no timing events)
int launch_solve_static(ddcca_ctx *ctx, const double *C11, const double *C22, const double *Cw, const double *CT,
                        int k, int L, double ridge, float *W1, float *W2, double *rho);
int static_solve_flags(ddcca_ctx *ctx, int host[4]);
int launch_conv(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L,
                float *out);
// the same with three-piece bf16 operands (DDCCA_CONV_BF16X3)
int launch_conv_split(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L,
                      float *out);
// output for map n goes to element (n / group) * group_stride + (n % group) * A * bins of `out`,
// whose element type out_type (DDCCA_FEAT_*) selects
int launch_hash_hist(ddcca_ctx *ctx, const float *maps, int64_t n, int L2, int h, int w, int bh, int bw,
                     int sy, int sx, void *out, int out_type, int64_t group, int64_t group_stride);

// information-quality table of the output layer (device, owned by the context): lut[c] = log(total) -
// log(c + 1), total = bh*bw + 2^L2, for c < lut_n; all three outputs are zero for the count output
int prepare_iq_table(ddcca_ctx *ctx, int out_type, int bh, int bw, int L2, const float **lut, int *lut_n,
                     double *log_total);
// stage convolution of n input maps with the L2 filters W fused with hashing + block histograms: the
// the fused last stage in two kernels when the convolution runs on three-piece operands: the convolution writes
// the hash codes of its (at most 8) maps, one byte per pixel, and the histograms are counted from those
int launch_conv_split_codes(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L,
                            unsigned char *codes);
int launch_code_hist(ddcca_ctx *ctx, const unsigned char *codes, int64_t n, int L2, int h, int w, int bh, int bw,
                     int sy, int sx, void *out, int out_type, int64_t group, int64_t group_stride);
// same output as launch_conv followed by launch_hash_hist, without the maps in between
int launch_conv_hash_hist(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L2,
                          int bh, int bw, int sy, int sx, void *out, int out_type, int64_t group,
                          int64_t group_stride);

}  // namespace ddcca
