// Packing of mixed-precision rows (Sec. 4.2 last paragraph and App. D.2: rows of
// equal bit width are gathered and processed together; Sec. 5.4: centroids are
// stored in lower precision).  Two kernels: a one-workgroup plan that orders the
// rows by (bits, row index) and lays out the groups, and a row kernel that
// rebuilds each label from the cluster thresholds and emits the bit stream
// (32 columns = b whole words per thread, assembled in registers).
#include "skim_common.h"

#include <hip/hip_fp16.h>
#include <math.h>

#include <mutex>

namespace {

constexpr int SKIM_PACK_STATIC_MAX_DEVICES = 64;
constexpr int PLAN_THREADS = 1024;
constexpr int PACK_THREADS = 256;

struct PackPlan {         // lives in the workspace
    long long row_start[6];   // first packed position of the b-bit group
    long long word_start[6];  // == group_word_offset
    long long cb_start[6];    // first codebook entry of the group
};

__global__ void __launch_bounds__(PLAN_THREADS) pack_plan_kernel(long long n, long long m, const uint8_t *bits,
                                                                 int *rowpos, int *row_perm, PackPlan *plan,
                                                                 long long *group_word_offset) {
    __shared__ int cnt[4][PLAN_THREADS];
    __shared__ long long gstart[6];
    const int t = threadIdx.x;
    const long long per = (n + PLAN_THREADS - 1) / PLAN_THREADS;
    const long long i0 = per * t, i1 = min(n, i0 + per);
    int c[4] = {0, 0, 0, 0};
    for (long long i = i0; i < i1; ++i) {
        const int b = bits[i];
        if (b >= 1 && b <= 4) c[b - 1]++;
    }
    for (int b = 0; b < 4; ++b) cnt[b][t] = c[b];
    __syncthreads();
    // exclusive scan of each bit width's counts over the threads (one wavefront per bit width)
    const int wave = t >> 6, lane = t & 63;
    if (wave < 4) {
        int run = 0;
        for (int base = 0; base < PLAN_THREADS; base += 64) {
            const int v = cnt[wave][base + lane];
            int inc = v;
            for (int d = 1; d < 64; d <<= 1) {
                const int u = __shfl_up(inc, d, 64);
                if (lane >= d) inc += u;
            }
            cnt[wave][base + lane] = run + inc - v;
            run += __shfl(inc, 63, 64);
        }
        if (lane == 0) gstart[wave + 1] = run;  // group sizes for now
    }
    __syncthreads();
    if (t == 0) {
        long long rows = 0, words = 0, cbs = 0;
        plan->row_start[0] = plan->word_start[0] = plan->cb_start[0] = 0;
        group_word_offset[0] = 0;
        for (int b = 1; b <= 4; ++b) {
            const long long sz = gstart[b];
            plan->row_start[b] = rows;
            plan->word_start[b] = words;
            plan->cb_start[b] = cbs;
            group_word_offset[b] = words;
            gstart[b] = rows;
            rows += sz;
            words += sz * ((m * b + 31) / 32);
            cbs += sz * (1ll << b);
        }
        plan->row_start[5] = rows;
        plan->word_start[5] = words;
        plan->cb_start[5] = cbs;
        group_word_offset[5] = words;
    }
    __syncthreads();
    long long pos[4];
    for (int b = 0; b < 4; ++b) pos[b] = gstart[b + 1] + cnt[b][t];
    for (long long i = i0; i < i1; ++i) {
        const int b = bits[i];
        if (b >= 1 && b <= 4) {
            const long long p = pos[b - 1]++;
            rowpos[i] = (int)p;
            row_perm[p] = (int)i;
        } else {
            rowpos[i] = -1;
        }
    }
}

// One workgroup per row.  A thread takes 32 consecutive columns at a time: their B-bit labels fill
// exactly B words, assembled in registers and stored without staging (no LDS traffic, no barriers
// inside the row).  ALPHA / DW: the call scales the columns / wants the residual; a group that lies
// wholly inside the row (all but the last one) takes the path without per-column bounds.
template <int B, bool ALPHA, bool DW>
__device__ __forceinline__ void pack_row_body(const float *__restrict__ Wr, const float *__restrict__ alpha, uint32_t m,
                                              const float *thr, const int *thl, const float *cbf,
                                              uint32_t *__restrict__ out_words, uint32_t wpr, float *__restrict__ dWr) {
    const uint32_t ngroups = (m + 31u) >> 5;
    const bool vec_ok = ((((uintptr_t)Wr) | (ALPHA ? (uintptr_t)alpha : 0) | (DW ? (uintptr_t)dWr : 0)) & 15) == 0;
    for (uint32_t g = threadIdx.x; g < ngroups; g += PACK_THREADS) {
        const uint32_t j0 = g << 5;
        const uint32_t valid = min(32u, m - j0);
        const bool full = valid == 32u && vec_ok;
        float w[32], a[32];
        if (full) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const float4 v = *(const float4 *)(Wr + j0 + 4 * q);
                w[4 * q] = v.x; w[4 * q + 1] = v.y; w[4 * q + 2] = v.z; w[4 * q + 3] = v.w;
                if (ALPHA) {
                    const float4 u = *(const float4 *)(alpha + j0 + 4 * q);
                    a[4 * q] = u.x; a[4 * q + 1] = u.y; a[4 * q + 2] = u.z; a[4 * q + 3] = u.w;
                }
            }
        } else {
#pragma unroll
            for (int jj = 0; jj < 32; ++jj) {
                w[jj] = ((uint32_t)jj < valid) ? Wr[j0 + jj] : 0.0f;
                if (ALPHA) a[jj] = ((uint32_t)jj < valid) ? alpha[j0 + jj] : 1.0f;
            }
        }
        uint32_t words[B + 1];
#pragma unroll
        for (int k = 0; k <= B; ++k) words[k] = 0u;
        float dq[32];
#pragma unroll
        for (int jj = 0; jj < 32; ++jj) {
            const float wt = ALPHA ? __fdiv_rn(w[jj], a[jj]) : w[jj];
            // first position whose bound is >= wt (binary search over the sorted bounds, +inf beyond the 2^B-th)
            int pos = 0;
            if (B >= 4) pos = (thr[7] < wt) ? 8 : 0;
            if (B >= 3) pos += (thr[pos + 3] < wt) ? 4 : 0;
            if (B >= 2) pos += (thr[pos + 1] < wt) ? 2 : 0;
            pos += (thr[pos] < wt) ? 1 : 0;
            uint32_t l = (uint32_t)thl[pos];
            if (DW) dq[jj] = __fmaf_rn(ALPHA ? -a[jj] : -1.0f, cbf[l], w[jj]);
            if (!full) l = ((uint32_t)jj < valid) ? l : 0u;            // padding bits stay zero
            const int bit = jj * B, wi = bit >> 5, sh = bit & 31;
            words[wi] |= l << sh;
            if (sh + B > 32) words[wi + 1] |= l >> (32 - sh);
        }
#pragma unroll
        for (int k = 0; k < B; ++k)
            if (g * B + k < wpr) out_words[g * B + k] = words[k];
        if (DW) {
            if (full) {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    *(float4 *)(dWr + j0 + 4 * q) = make_float4(dq[4 * q], dq[4 * q + 1], dq[4 * q + 2], dq[4 * q + 3]);
            } else {
#pragma unroll
                for (int jj = 0; jj < 32; ++jj)
                    if ((uint32_t)jj < valid) dWr[j0 + jj] = dq[jj];
            }
        }
    }
}

template <int B>
__device__ __forceinline__ void pack_row_dispatch(const float *Wr, const float *alpha, uint32_t m, const float *thr,
                                                  const int *thl, const float *cbf, uint32_t *ow, uint32_t wpr, float *dWr) {
    if (alpha) {
        if (dWr) pack_row_body<B, true, true>(Wr, alpha, m, thr, thl, cbf, ow, wpr, dWr);
        else pack_row_body<B, true, false>(Wr, alpha, m, thr, thl, cbf, ow, wpr, dWr);
    } else {
        if (dWr) pack_row_body<B, false, true>(Wr, alpha, m, thr, thl, cbf, ow, wpr, dWr);
        else pack_row_body<B, false, false>(Wr, alpha, m, thr, thl, cbf, ow, wpr, dWr);
    }
}

__global__ void __launch_bounds__(PACK_THREADS) pack_rows_kernel(const float *W, const float *alpha, long long m,
                                                                 long long ld, const uint8_t *bits,
                                                                 const double *cent, const float *upper,
                                                                 const int *rowpos, const PackPlan *plan,
                                                                 uint32_t *codes, uint16_t *codebooks, float *dW) {
    __shared__ float thr[16];
    __shared__ int thl[16];
    __shared__ float cbf[16];
    const long long row = blockIdx.x;
    const int tid = threadIdx.x;
    const int p = rowpos[row];
    if (p < 0) return;  // bits outside 1..4: row is not part of the packed model
    const int b = bits[row];
    const int K = 1 << b;
    const long long wpr = (m * b + 31) / 32;
    const long long local = (long long)p - plan->row_start[b];
    const long long word0 = plan->word_start[b] + local * wpr;
    const long long cb0 = plan->cb_start[b] + local * K;

    if (tid < 16) {
        thr[tid] = INFINITY;
        thl[tid] = 0;
    }
    __syncthreads();
    if (tid < K) {
        const float up = upper[row * 16 + tid];
        int rank = 0;
        for (int j = 0; j < K; ++j) {
            const float uj = upper[row * 16 + j];
            rank += (uj < up || (uj == up && j < tid)) ? 1 : 0;
        }
        thr[rank] = up;
        thl[rank] = tid;
        const __half h = __float2half_rn((float)cent[row * 16 + tid]);
        codebooks[cb0 + tid] = __half_as_ushort(h);
        cbf[tid] = __half2float(h);
    }
    __syncthreads();
    // thr[0..K) ascending (empty clusters, -inf, first), +inf beyond; a value above every bound
    // (cannot happen for thresholds taken from this row) falls to the cluster of the largest bound
    if (tid >= K && tid < 16) thl[tid] = thl[K - 1];
    __syncthreads();
    const float *Wr = W + row * ld;
    float *dWr = dW ? dW + row * m : nullptr;
    uint32_t *ow = codes + word0;
    switch (b) {
        case 1: pack_row_dispatch<1>(Wr, alpha, (uint32_t)m, thr, thl, cbf, ow, (uint32_t)wpr, dWr); break;
        case 2: pack_row_dispatch<2>(Wr, alpha, (uint32_t)m, thr, thl, cbf, ow, (uint32_t)wpr, dWr); break;
        case 3: pack_row_dispatch<3>(Wr, alpha, (uint32_t)m, thr, thl, cbf, ow, (uint32_t)wpr, dWr); break;
        default: pack_row_dispatch<4>(Wr, alpha, (uint32_t)m, thr, thl, cbf, ow, (uint32_t)wpr, dWr); break;
    }
}

}  // namespace

// The two launches of a pack call; rowpos (n ints) and plan are the call's scratch.
static skim_status launch_pack(skim_ctx *ctx, const float *W, const float *alpha, int64_t n, int64_t m, int64_t ld,
                               const uint8_t *bits, const double *centroids, const float *upper, uint32_t *codes,
                               int64_t *group_word_offset, int32_t *row_perm, uint16_t *codebooks_fp16, float *dW,
                               int *rowpos, PackPlan *plan) {
    hipLaunchKernelGGL(pack_plan_kernel, dim3(1), dim3(PLAN_THREADS), 0, ctx->stream, (long long)n, (long long)m, bits,
                       rowpos, row_perm, plan, (long long *)group_word_offset);
    SKIM_HIP(ctx, hipGetLastError());
    hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)n), dim3(PACK_THREADS), 0, ctx->stream, W, alpha, (long long)m,
                       (long long)ld, bits, centroids, upper, rowpos, plan, codes, codebooks_fp16, dW);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}

static skim_status check_pack_args(skim_ctx *ctx, const float *W, int64_t n, int64_t m, int64_t ld, const uint8_t *bits,
                                   const double *centroids, const float *upper, uint32_t *codes,
                                   int64_t *group_word_offset, int32_t *row_perm, uint16_t *codebooks_fp16) {
    if (!W || !bits || !centroids || !upper || !codes || !group_word_offset || !row_perm || !codebooks_fp16)
        SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_pack: NULL argument");
    if (n < 1 || n > 0x7fffffff || m < 1 || ld < m) SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "skim_pack: bad shape n=%lld m=%lld ld=%lld", (long long)n, (long long)m, (long long)ld);
    if (m >= (1ll << 29)) SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "skim_pack: row too long (m < 2^29)");
    return SKIM_OK;
}

extern "C" skim_status skim_pack(skim_ctx *ctx, const float *W, const float *alpha, int64_t n, int64_t m,
                                 int64_t ld, const uint8_t *bits, const double *centroids, const float *upper,
                                 uint32_t *codes, int64_t *group_word_offset, int32_t *row_perm,
                                 uint16_t *codebooks_fp16, float *dW) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if ((st = check_pack_args(ctx, W, n, m, ld, bits, centroids, upper, codes, group_word_offset, row_perm,
                              codebooks_fp16)) != SKIM_OK)
        return st;
    skim_ws_cursor cur{(char *)ctx->ws, 0, ctx->ws_bytes};
    int *rowpos = (int *)cur.take((size_t)n * sizeof(int));
    PackPlan *plan = (PackPlan *)cur.take(sizeof(PackPlan));
    if (!rowpos || !plan) SKIM_FAIL(ctx, SKIM_ERR_WORKSPACE, "skim_pack: workspace missing or smaller than skim_workspace_bytes(n, m)");
    return launch_pack(ctx, W, alpha, n, m, ld, bits, centroids, upper, codes, group_word_offset, row_perm,
                       codebooks_fp16, dW, rowpos, plan);
}

// ---------------------------------------------------------------------------------------------
// skim_pack for callers that cannot allocate device memory or register a workspace: the scratch of
// the call (row positions and the group table) lives in a file-scope device array.  Every device the
// library runs on holds its own copy of the array at its own address; the address is looked up once
// per device by skim_create (through skim_pack_static_setup below, with that device current) and
// kept in the context.  Host code never passes the array's name to a kernel: on the host the name
// is only a handle for hipGetSymbolAddress.
// ---------------------------------------------------------------------------------------------
static_assert(sizeof(PackPlan) <= 256, "the group table must fit the first 256 bytes of the static scratch");
static __device__ __align__(256) unsigned char pack_static_scratch[SKIM_PACK_STATIC_MAX_ROWS * sizeof(int) + 256];

static std::mutex pack_static_mutex;
static void *pack_static_addr[SKIM_PACK_STATIC_MAX_DEVICES];   // per device, looked up once

skim_status skim_pack_static_setup(skim_ctx *ctx) {
    if (ctx->device < 0 || ctx->device >= SKIM_PACK_STATIC_MAX_DEVICES)
        SKIM_FAIL(ctx, SKIM_ERR_ARG, "device %d beyond the %d devices the static scratch table holds", ctx->device,
                  SKIM_PACK_STATIC_MAX_DEVICES);
    std::lock_guard<std::mutex> lock(pack_static_mutex);
    if (!pack_static_addr[ctx->device]) {
        void *ptr = nullptr;
        SKIM_HIP(ctx, hipGetSymbolAddress(&ptr, HIP_SYMBOL(pack_static_scratch)));
        if (!ptr) SKIM_FAIL(ctx, SKIM_ERR_HIP, "hipGetSymbolAddress returned no address for the static pack scratch");
        pack_static_addr[ctx->device] = ptr;
    }
    ctx->pack_scratch = pack_static_addr[ctx->device];
    return SKIM_OK;
}

extern "C" skim_status skim_pack_static(skim_ctx *ctx, const float *W, const float *alpha, int64_t n, int64_t m,
                                        int64_t ld, const uint8_t *bits, const double *centroids,
                                        const float *upper, uint32_t *codes, int64_t *group_word_offset,
                                        int32_t *row_perm, uint16_t *codebooks_fp16, float *dW) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if ((st = check_pack_args(ctx, W, n, m, ld, bits, centroids, upper, codes, group_word_offset, row_perm,
                              codebooks_fp16)) != SKIM_OK)
        return st;
    if (n > SKIM_PACK_STATIC_MAX_ROWS)
        SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "skim_pack_static: n = %lld rows, the static scratch holds %d at most (use skim_pack)",
                  (long long)n, SKIM_PACK_STATIC_MAX_ROWS);
    if (!ctx->pack_scratch) SKIM_FAIL(ctx, SKIM_ERR_HIP, "skim_pack_static: the context has no static scratch address");
    // layout: the group table in the first 256 bytes, then one int per row.  Both are written in full by the
    // plan kernel before the row kernel reads them, so nothing of an earlier call survives into this one.
    PackPlan *plan = (PackPlan *)ctx->pack_scratch;
    int *rowpos = (int *)((char *)ctx->pack_scratch + 256);
    return launch_pack(ctx, W, alpha, n, m, ld, bits, centroids, upper, codes, group_word_offset, row_perm,
                       codebooks_fp16, dW, rowpos, plan);
}
