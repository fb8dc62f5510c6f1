// Internal declarations shared by the translation units of libskim (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "skim.h"

struct skim_ctx {
    int device;
    hipStream_t stream;
    void *ws;
    size_t ws_bytes;
    int lds_limit;      // max LDS bytes one workgroup may use on this device
    int num_cu;
    char err[512];
    // optional per-kernel timing of the clustering calls (skim_profile_enable)
    int profiling;
    hipEvent_t ev[3];    // before sort, between sort and Lloyd, after Lloyd
    int ev_valid;
    size_t sort_lds_enabled[4];   // dynamic LDS size each variant of the sort kernel has been allowed so far (through this context)
    int greedy_lds_enabled, xtx_lds_enabled, gemm3_lds_enabled;   // the larger dynamic-LDS limit of these kernels has been set through this context
    int validate;        // check W, S, alpha of the clustering calls for values the method is not defined on
    void *pack_scratch;  // this device's address of the static scratch of skim_pack_static
    int *sort_counters;  // device memory owned by the context: [0] units of work handed out by the running sort_kernel, [1] its workgroups
                         // that are done; both are zero between launches (the last workgroup to finish clears them)
};

#define SKIM_FAIL(ctx, code, ...)                                   \
    do {                                                            \
        snprintf((ctx)->err, sizeof((ctx)->err), __VA_ARGS__);      \
        return (code);                                              \
    } while (0)

#define SKIM_HIP(ctx, call)                                                                  \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess)                                                                \
            SKIM_FAIL(ctx, SKIM_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_));     \
    } while (0)

// Makes `device` current for the calling thread; returns SKIM_ERR_HIP on failure.
static inline skim_status skim_enter(skim_ctx *ctx) {
    if (!ctx) return SKIM_ERR_ARG;
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) SKIM_FAIL(ctx, SKIM_ERR_HIP, "hipSetDevice failed: %s", hipGetErrorString(e));
    ctx->err[0] = 0;
    return SKIM_OK;
}

// Workspace carving: 256-byte aligned pieces of the registered buffer.
struct skim_ws_cursor {
    char *base;
    size_t off, cap;
    void *take(size_t bytes) {
        size_t a = (off + 255) & ~(size_t)255;
        if (a + bytes > cap) return nullptr;
        off = a + bytes;
        return base + a;
    }
};

static inline int skim_block_offset(int bmin, int b) {  // start of block b inside a row of the *_all arrays
    return (1 << b) - (1 << bmin);
}

// Looks up this device's address of the static scratch of skim_pack_static (the device must be current).
skim_status skim_pack_static_setup(skim_ctx *ctx);

// skim_layer_loss with the per-row losses written at a stride (row i at row_loss[i * row_stride]).  kept (may be
// NULL): kept_n centroids per row at kept + i * kept_stride, used for clusters whose members carry no mass.
skim_status skim_layer_loss_strided(skim_ctx *ctx, const float *W, const float *S, const float *alpha, const float *H,
                                    int64_t n, int64_t m, int64_t ld, const uint8_t *labels, double *loss,
                                    double *row_loss, int64_t row_stride, const double *kept, int64_t kept_stride,
                                    int kept_n);
