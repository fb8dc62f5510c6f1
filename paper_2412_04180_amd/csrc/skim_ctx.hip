// Context, workspace registration and error text of libskim.
#include "skim_common.h"

static char g_create_err[512] = "";

extern "C" skim_status skim_create(skim_ctx **out, int device, void *hip_stream) {
    if (!out) {
        snprintf(g_create_err, sizeof(g_create_err), "skim_create: out is NULL");
        return SKIM_ERR_ARG;
    }
    *out = nullptr;
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess || count <= 0) {
        snprintf(g_create_err, sizeof(g_create_err), "skim_create: no HIP device (%s)",
                 e == hipSuccess ? "count is 0" : hipGetErrorString(e));
        return SKIM_ERR_HIP;
    }
    if (device < 0 || device >= count) {
        snprintf(g_create_err, sizeof(g_create_err), "skim_create: device %d out of range [0,%d)", device, count);
        return SKIM_ERR_ARG;
    }
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) {
        snprintf(g_create_err, sizeof(g_create_err), "skim_create: hipGetDeviceProperties: %s", hipGetErrorString(e));
        return SKIM_ERR_HIP;
    }
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
        snprintf(g_create_err, sizeof(g_create_err),
                 "skim_create: device %d is %s; this library is built for gfx950 only", device, prop.gcnArchName);
        return SKIM_ERR_HIP;
    }
    e = hipSetDevice(device);
    if (e != hipSuccess) {
        snprintf(g_create_err, sizeof(g_create_err), "skim_create: hipSetDevice: %s", hipGetErrorString(e));
        return SKIM_ERR_HIP;
    }
    skim_ctx *c = new skim_ctx();
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    c->ws = nullptr;
    c->ws_bytes = 0;
    c->lds_limit = (int)prop.sharedMemPerBlock;
    int optin = 0;
    if (hipDeviceGetAttribute(&optin, hipDeviceAttributeMaxSharedMemoryPerBlock, device) == hipSuccess && optin > c->lds_limit)
        c->lds_limit = optin;
    if (c->lds_limit < 160 * 1024) {   // gfx950 has 160 KB per compute unit; the row sort is laid out for it
        snprintf(g_create_err, sizeof(g_create_err),
                 "skim_create: device %d reports %d bytes of LDS per workgroup, the row sort needs %d", device,
                 c->lds_limit, 160 * 1024);
        delete c;
        return SKIM_ERR_HIP;
    }
    c->num_cu = prop.multiProcessorCount;
    c->profiling = 0;
    c->ev_valid = 0;
    for (int i = 0; i < 3; ++i) c->ev[i] = nullptr;
    c->err[0] = 0;
    for (int i = 0; i < 4; ++i) c->sort_lds_enabled[i] = 0;
    c->greedy_lds_enabled = 0;
    c->xtx_lds_enabled = 0;
    c->gemm3_lds_enabled = 0;
    c->validate = 0;
    c->pack_scratch = nullptr;
    c->sort_counters = nullptr;
    e = hipMalloc((void **)&c->sort_counters, 256);
    if (e == hipSuccess) e = hipMemset(c->sort_counters, 0, 256);
    if (e == hipSuccess) e = hipDeviceSynchronize();   // the clear is complete before any stream of the caller's uses the context
    if (e != hipSuccess) {
        snprintf(g_create_err, sizeof(g_create_err), "skim_create: the sort's work counters: %s", hipGetErrorString(e));
        if (c->sort_counters) (void)hipFree(c->sort_counters);
        delete c;
        return SKIM_ERR_HIP;
    }
    if (skim_pack_static_setup(c) != SKIM_OK) {
        snprintf(g_create_err, sizeof(g_create_err), "skim_create: %s", c->err);
        (void)hipFree(c->sort_counters);
        delete c;
        return SKIM_ERR_HIP;
    }
    *out = c;
    return SKIM_OK;
}

extern "C" skim_status skim_destroy(skim_ctx *ctx) {
    if (!ctx) return SKIM_ERR_ARG;
    for (int i = 0; i < 3; ++i)
        if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
    if (ctx->sort_counters) (void)hipFree(ctx->sort_counters);
    delete ctx;
    return SKIM_OK;
}

extern "C" skim_status skim_validate_enable(skim_ctx *ctx, int on) {
    if (!ctx) return SKIM_ERR_ARG;
    ctx->validate = on ? 1 : 0;
    return SKIM_OK;
}

extern "C" skim_status skim_profile_enable(skim_ctx *ctx, int on) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (on && !ctx->ev[0]) {
        for (int i = 0; i < 3; ++i) SKIM_HIP(ctx, hipEventCreate(&ctx->ev[i]));
    }
    ctx->profiling = on ? 1 : 0;
    ctx->ev_valid = 0;
    return SKIM_OK;
}

extern "C" skim_status skim_profile_last(skim_ctx *ctx, float *sort_ms, float *lloyd_ms) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!ctx->profiling || !ctx->ev_valid) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_profile_last: no timed clustering call yet");
    SKIM_HIP(ctx, hipEventSynchronize(ctx->ev[2]));
    float a = 0.f, b = 0.f;
    SKIM_HIP(ctx, hipEventElapsedTime(&a, ctx->ev[0], ctx->ev[1]));
    SKIM_HIP(ctx, hipEventElapsedTime(&b, ctx->ev[1], ctx->ev[2]));
    if (sort_ms) *sort_ms = a;
    if (lloyd_ms) *lloyd_ms = b;
    return SKIM_OK;
}

extern "C" const char *skim_last_error(const skim_ctx *ctx) { return ctx ? ctx->err : g_create_err; }

extern "C" size_t skim_workspace_bytes(int64_t n, int64_t m) {
    if (n < 0 || m < 0) return 0;
    const size_t N = (size_t)n, M = (size_t)m;
    const size_t ntile = (M + 127) / 128, nstrip = (N + 7) / 8;
    size_t b = 0;
    b += 3 * N * M * sizeof(uint16_t) + N * M * sizeof(float);   // scale step: dW (as three bfloat16 pieces per value, or as float32) and P
    b += 3 * M * M * sizeof(uint16_t);   // the pieces of H
    b += 2 * N * 16 * sizeof(double);    // centroids and masses from fixed labels
    b += ntile * N * sizeof(double);     // per-tile row sums of the loss
    b += nstrip * M * sizeof(double);    // per-strip column sums of the gradient
    b += N * 30 * sizeof(double);        // centroid scratch of skim_error_table when the caller wants none
    b += N * (14 * M + 8192);            // clustering: sorted keys (8 B per weight), per-chunk sums and Lloyd state between the kernels
    if (M > 16384) b += N * 8 * M + N * 8 + 256;   // rows sorted in two halves: the unmerged keys, a mass flag per half
    b += N * sizeof(int) + 1024;         // pack: row positions and group table
    b += N * 4 * sizeof(double) + 1024;  // L-full error table: S-diag errors and the loss scalar at the tail
    b += N * (16 * sizeof(float) + sizeof(double)) + 1024;   // scale training: thresholds and errors of the re-clustering
    return b + 16 * 256;                 // alignment slack (every piece is 256-byte aligned)
}

extern "C" skim_status skim_set_workspace(skim_ctx *ctx, void *dev_ptr, size_t bytes) {
    if (!ctx) return SKIM_ERR_ARG;
    if (dev_ptr && ((uintptr_t)dev_ptr & 255)) SKIM_FAIL(ctx, SKIM_ERR_ARG, "workspace must be 256-byte aligned");
    ctx->ws = dev_ptr;
    ctx->ws_bytes = dev_ptr ? bytes : 0;
    return SKIM_OK;
}
