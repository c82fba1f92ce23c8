// Drives the host side of the C ABI (argument validation, state checks, error texts, context life cycle) on a
// machine without a GPU, for a build of api.hip whose host code carries -fsanitize=address,undefined.  Every call
// below must return its documented error code without touching a device.  Prints "api sanitize ok".
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/ddcca.h"

static int failures = 0;
#define EXPECT(call, code)                                                                  \
    do {                                                                                    \
        const int rc__ = (call);                                                            \
        if (rc__ != (code)) {                                                               \
            printf("%s -> %d, expected %d\n", #call, rc__, (code));                         \
            ++failures;                                                                     \
        }                                                                                   \
    } while (0)

int main()
{
    ddcca_ctx *ctx = nullptr;
    EXPECT(ddcca_create(nullptr, 0, nullptr), DDCCA_EINVAL);
    EXPECT(ddcca_create(&ctx, -1, nullptr), DDCCA_EINVAL);
    EXPECT(ddcca_create(&ctx, 1 << 20, nullptr), DDCCA_EINVAL);
    EXPECT(ddcca_create(&ctx, 0, nullptr), DDCCA_OK);
    float *f = reinterpret_cast<float *>(0x1000);          // never dereferenced: validation comes first
    double *d = reinterpret_cast<double *>(0x1000);
    int32_t *c = reinterpret_cast<int32_t *>(0x1000);
    uint16_t *u = reinterpret_cast<uint16_t *>(0x1000);

    EXPECT(ddcca_corr_begin(ctx, 4, 2, 1, 8, 8), DDCCA_EINVAL);            // even k
    EXPECT(ddcca_corr_begin(ctx, 11, 2, 1, 8, 8), DDCCA_EINVAL);           // k too large
    EXPECT(ddcca_corr_begin(ctx, 5, 0, 1, 8, 8), DDCCA_EINVAL);
    EXPECT(ddcca_corr_begin(ctx, 5, 2, 0, 8, 8), DDCCA_EINVAL);
    EXPECT(ddcca_corr_begin(ctx, 5, 2, 1, 0, 8), DDCCA_EINVAL);
    EXPECT(ddcca_corr_begin(ctx, 5, 70000, 1, 8, 8), DDCCA_EINVAL);        // n_cls * G > 65535
    EXPECT(ddcca_corr_accumulate(ctx, f, f, c, 4), DDCCA_ESTATE);
    EXPECT(ddcca_corr_export(ctx, d, d, d, d, d), DDCCA_ESTATE);
    EXPECT(ddcca_solve_filters(ctx, 4, 1e-4, f, f, d), DDCCA_ESTATE);
    if (!strlen(ddcca_last_error(ctx))) { printf("empty error text\n"); ++failures; }

    EXPECT(ddcca_dcca_solve(ctx, d, d, d, d, 5, 0, 1e-4, f, f, d), DDCCA_EINVAL);
    EXPECT(ddcca_dcca_solve(ctx, d, d, d, d, 5, 25, 1e-4, f, f, d), DDCCA_EINVAL);
    EXPECT(ddcca_dcca_solve(ctx, d, d, d, d, 5, 4, 0.0, f, f, d), DDCCA_EINVAL);
    EXPECT(ddcca_dcca_solve(ctx, nullptr, d, d, d, 5, 4, 1e-4, f, f, d), DDCCA_EINVAL);
    EXPECT(ddcca_learn_stage_filters(ctx, f, f, c, 0, 1, 8, 8, 2, 5, 4, 1e-4, f, f, d), DDCCA_EINVAL);
    EXPECT(ddcca_learn_stage_filters(ctx, nullptr, f, c, 4, 1, 8, 8, 2, 5, 4, 1e-4, f, f, d), DDCCA_EINVAL);
    EXPECT(ddcca_learn_next_stage_filters(ctx, f, f, c, 4, 1, 8, 8, 2, f, f, 5, 25, 5, 4, 1e-4, 0, f, f, d),
           DDCCA_EINVAL);
    EXPECT(ddcca_learn_next_stage_filters(ctx, f, f, c, 4, 1, 8, 8, 2, f, f, 5, 4, 5, 4, 1e-4, -1, f, f, d),
           DDCCA_EINVAL);

    EXPECT(ddcca_apply_stage(ctx, f, -1, 8, 8, f, 5, 4, f), DDCCA_EINVAL);
    EXPECT(ddcca_apply_stage(ctx, f, 2, 8, 8, f, 5, 0, f), DDCCA_EINVAL);
    EXPECT(ddcca_apply_stage(ctx, f, 2, 8, 8, nullptr, 5, 4, f), DDCCA_EINVAL);
    EXPECT(ddcca_apply_stage(ctx, f, 0, 8, 8, f, 5, 4, f), DDCCA_OK);      // nothing to do
    EXPECT(ddcca_hash_histogram(ctx, f, 2, 13, 8, 8, 4, 4, 2, 2, u), DDCCA_EINVAL);
    EXPECT(ddcca_hash_histogram(ctx, f, 2, 8, 8, 8, 9, 4, 2, 2, u), DDCCA_EINVAL);
    EXPECT(ddcca_hash_histogram(ctx, f, 2, 8, 8, 8, 4, 4, 0, 2, u), DDCCA_EINVAL);
    EXPECT(ddcca_hash_histogram(ctx, f, 2, 8, 300, 300, 256, 257, 8, 8, u), DDCCA_EOVERFLOW);
    EXPECT(ddcca_hash_histogram(ctx, f, 0, 8, 8, 8, 4, 4, 2, 2, u), DDCCA_OK);
    EXPECT(ddcca_hash_iq(ctx, f, 2, 8, 8, 8, 4, 4, 2, 2, 9, u), DDCCA_EINVAL);
    EXPECT(ddcca_apply_stage_hash(ctx, f, 2, 8, 8, f, 6, 8, 4, 4, 2, 2, DDCCA_FEAT_COUNT_U16, u), DDCCA_EINVAL);

    ddcca_model model;
    memset(&model, 0, sizeof(model));
    model.k = 5; model.L1 = 4; model.L2 = 4; model.block_h = model.block_w = 4; model.stride_y = model.stride_x = 2;
    EXPECT(ddcca_extract_features(ctx, f, f, 2, 8, 8, nullptr, u), DDCCA_EINVAL);
    EXPECT(ddcca_extract_features(ctx, f, f, 2, 8, 8, &model, u), DDCCA_EINVAL);        // null filters
    for (int s = 0; s < 2; ++s)
        for (int v = 0; v < 2; ++v) model.W[s][v] = f;
    model.batch_images = -3;
    EXPECT(ddcca_extract_features_fused(ctx, f, f, 2, 8, 8, &model, DDCCA_FEAT_IQ_F16, u), DDCCA_EINVAL);
    model.batch_images = 0;
    EXPECT(ddcca_extract_iq_features(ctx, f, f, 0, 8, 8, &model, DDCCA_FEAT_IQ_F32, u), DDCCA_OK);

    EXPECT(ddcca_set_option(ctx, 99, 0), DDCCA_EINVAL);
    EXPECT(ddcca_set_option(ctx, DDCCA_OPT_CONV_ARITH, 7), DDCCA_EINVAL);
    EXPECT(ddcca_set_option(ctx, DDCCA_OPT_GRAM_ARITH, DDCCA_GRAM_LAG_FP32), DDCCA_OK);
    EXPECT(ddcca_set_option(ctx, DDCCA_OPT_GRAM_ARITH, DDCCA_GRAM_FP32), DDCCA_OK);
    EXPECT(ddcca_profile_enable(ctx, 1), DDCCA_OK);
    EXPECT(ddcca_profile_select(ctx, 0u), DDCCA_EINVAL);
    EXPECT(ddcca_profile_select(ctx, 1u << DDCCA_K_GRAM), DDCCA_OK);
    double ms = 0.0;
    int64_t n = 0;
    EXPECT(ddcca_profile_read(ctx, DDCCA_K_COUNT, &ms, &n), DDCCA_EINVAL);
    EXPECT(ddcca_profile_read(ctx, DDCCA_K_GRAM, &ms, &n), DDCCA_OK);
    EXPECT(ddcca_profile_reset(ctx), DDCCA_OK);
    ddcca_destroy(ctx);
    ddcca_destroy(nullptr);
    if (failures) return 1;
    printf("api sanitize ok\n");
    return 0;
}
