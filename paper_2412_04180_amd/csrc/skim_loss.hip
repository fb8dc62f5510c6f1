// placeholder until the contraction kernels land
#include "skim_common.h"
extern "C" skim_status skim_layer_loss(skim_ctx *ctx, const float *, const float *, const float *, const float *, int64_t,
                                       int64_t, int64_t, const uint8_t *, double *, double *) {
    if (!ctx) return SKIM_ERR_ARG;
    SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_layer_loss: not built yet");
}
extern "C" skim_status skim_scale_step(skim_ctx *ctx, const float *, const float *, const float *, int64_t, int64_t,
                                       int64_t, const uint8_t *, float *, float *, float *, int64_t,
                                       const skim_adam_opts *, double *, float *) {
    if (!ctx) return SKIM_ERR_ARG;
    SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_scale_step: not built yet");
}
