// Packing of mixed-precision rows (Sec. 4.2 last paragraph and App. D.2: rows of
// equal bit width are gathered and processed together; Sec. 5.4: centroids are
// stored in lower precision).  Two kernels: a one-workgroup plan that orders the
// rows by (bits, row index) and lays out the groups, and a row kernel that
// rebuilds each label from the cluster thresholds and emits the bit stream
// (32 columns = b whole words per four lanes, assembled in registers).
#include "skim_common.h"

#include <hip/hip_fp16.h>
#include <math.h>

#include <mutex>

namespace {

constexpr int SKIM_PACK_STATIC_MAX_DEVICES = 64;
constexpr int PLAN_THREADS = 1024;
constexpr int PACK_THREADS = 256;
constexpr int PACK_UNROLL = 1;   // groups of 32 columns a quad of lanes has in flight at a time; more of them cost
                                 // registers, and resident wavefronts hide the load latency better (measured: 48, 57,
                                 // 67 us per call on 4096 x 11008 with 1, 2, 3)

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
    // exclusive scan of each bit width's counts over the threads: one wavefront per bit width, a lane takes
    // PLAN_THREADS / 64 consecutive entries and the lanes' totals are scanned inside the VALU (DPP)
    const int wave = t >> 6, lane = t & 63;
    if (wave < 4) {
        constexpr int PER = PLAN_THREADS / 64;
        int v[PER];
        int tot = 0;
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            v[k] = cnt[wave][lane * PER + k];
            tot += v[k];
        }
        int inc = tot;
        inc += __builtin_amdgcn_update_dpp(0, inc, 0x111, 0xF, 0xF, false);   // row_shr:1
        inc += __builtin_amdgcn_update_dpp(0, inc, 0x112, 0xF, 0xF, false);   // row_shr:2
        inc += __builtin_amdgcn_update_dpp(0, inc, 0x114, 0xF, 0xF, false);   // row_shr:4
        inc += __builtin_amdgcn_update_dpp(0, inc, 0x118, 0xF, 0xF, false);   // row_shr:8
        inc += __builtin_amdgcn_update_dpp(0, inc, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1, 3
        inc += __builtin_amdgcn_update_dpp(0, inc, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2, 3
        int run = inc - tot;
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            cnt[wave][lane * PER + k] = run;
            run += v[k];
        }
        if (lane == 63) gstart[wave + 1] = inc;  // group sizes for now
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

// One workgroup per row.  Four neighbouring lanes take 32 consecutive columns, 8 each (two 16-byte loads per
// lane, a quad reads one 128-byte line): the B-bit labels of the 32 columns fill exactly B words.  A lane packs
// its 8 labels into 8 B bits and shifts them to their place in the B words; the four lanes OR their words
// together (DPP inside the quad) and lanes 0 .. B-1 of the quad store one word each, so a wavefront's stores are
// consecutive words.
// Label of a weight = cluster at position (number of the row's sorted cluster bounds below the weight).  The
// bounds are the same for the whole workgroup: they are read once into scalar registers and every weight is
// compared against them there (no dependent LDS lookups per weight); for 16 clusters, three scalar bounds pick a
// quarter and one 16-byte LDS read brings that quarter's bounds.  ident: positions and cluster indices coincide
// (centroids ascending in the cluster index, the usual case), so no position -> cluster lookup is needed.
// A lane works on PACK_UNROLL groups at a time (a "round": all their loads are in flight together); the loads of
// the first round are issued by the kernel before it sorts the bounds.  ALPHA / DW: the call scales the columns / wants the residual.
struct PackRound {
    float w[PACK_UNROLL][8], a[PACK_UNROLL][8];
};

template <bool ALPHA>
__device__ __forceinline__ void pack_load_round(PackRound &r, const float *__restrict__ Wr, const float *__restrict__ alpha,
                                                uint32_t m, uint32_t g0, bool vec_ok) {
    const uint32_t ngroups = (m + 31u) >> 5;
    const uint32_t t = threadIdx.x & 3u;
#pragma unroll
    for (int u = 0; u < PACK_UNROLL; ++u) {
        const uint32_t g = g0 + u * (PACK_THREADS / 4);
        const uint32_t j0 = (g << 5) + 8u * t;
        if (g >= ngroups) continue;
        if (vec_ok && j0 + 8u <= m) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const float4 v = *(const float4 *)(Wr + j0 + 4 * q);
                r.w[u][4 * q] = v.x; r.w[u][4 * q + 1] = v.y; r.w[u][4 * q + 2] = v.z; r.w[u][4 * q + 3] = v.w;
                if (ALPHA) {
                    const float4 x = *(const float4 *)(alpha + j0 + 4 * q);
                    r.a[u][4 * q] = x.x; r.a[u][4 * q + 1] = x.y; r.a[u][4 * q + 2] = x.z; r.a[u][4 * q + 3] = x.w;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                r.w[u][i] = (j0 + i < m) ? Wr[j0 + i] : 0.0f;
                if (ALPHA) r.a[u][i] = (j0 + i < m) ? alpha[j0 + i] : 1.0f;
            }
        }
    }
}

// cur: the first round, already loaded (pack_load_round at g0 = threadIdx.x / 4)
template <int B, bool ALPHA, bool DW>
__device__ __forceinline__ void pack_row_body(PackRound &cur, const float *__restrict__ Wr, const float *__restrict__ alpha,
                                              uint32_t m, bool vec_ok, const float *thr, const int *thl, const float *cbf,
                                              uint32_t *__restrict__ out_words, uint32_t wpr, float *__restrict__ dWr) {
    constexpr int K = 1 << B;
    constexpr int NSC = (B == 4) ? 3 : K - 1;      // bounds held in scalar registers
    float ts[NSC];
#pragma unroll
    for (int k = 0; k < NSC; ++k) {
        const float x = (B == 4) ? thr[4 * k + 3] : thr[k];
        ts[k] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x)));
    }
    int same = 1;
#pragma unroll
    for (int k = 0; k < K; ++k) same &= (thl[k] == k) ? 1 : 0;
    const bool ident = __builtin_amdgcn_readfirstlane(same) != 0;

    const uint32_t ngroups = (m + 31u) >> 5;
    const uint32_t t = threadIdx.x & 3u;
    // place of this lane's 8 B bits inside the B words of its group
    const uint32_t o = 8u * B * t, wi = o >> 5, sh = o & 31u;
    constexpr uint32_t GSTEP = PACK_THREADS / 4, RSTEP = PACK_UNROLL * GSTEP;
    for (uint32_t g0 = threadIdx.x >> 2; g0 < ngroups; g0 += RSTEP) {
        if (g0 != (threadIdx.x >> 2)) pack_load_round<ALPHA>(cur, Wr, alpha, m, g0, vec_ok);
#pragma unroll
        for (int u = 0; u < PACK_UNROLL; ++u) {
            const uint32_t g = g0 + u * GSTEP;
            const uint32_t j0 = (g << 5) + 8u * t;
            if (g >= ngroups) continue;          // (the same for the four lanes of a quad)
            const bool full = vec_ok && j0 + 8u <= m;
            uint32_t p = 0u;
            float dq[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float wt = ALPHA ? __fdiv_rn(cur.w[u][i], cur.a[u][i]) : cur.w[u][i];
                // first position whose bound is >= wt = number of bounds below wt (bounds ascending, +inf beyond the 2^B-th)
                uint32_t pos = 0u;
                if (B == 4) {
                    uint32_t q = 0u;
#pragma unroll
                    for (int k = 0; k < 3; ++k) q += (ts[k] < wt) ? 1u : 0u;
                    const float4 t4 = *(const float4 *)(thr + 4u * q);
                    pos = 4u * q + ((t4.x < wt) ? 1u : 0u) + ((t4.y < wt) ? 1u : 0u) + ((t4.z < wt) ? 1u : 0u);
                } else {
#pragma unroll
                    for (int k = 0; k < NSC; ++k) pos += (ts[k] < wt) ? 1u : 0u;
                }
                uint32_t l = ident ? pos : (uint32_t)thl[pos];
                if (DW) dq[i] = __fmaf_rn(ALPHA ? -cur.a[u][i] : -1.0f, cbf[l], cur.w[u][i]);
                if (!full) l = (j0 + i < m) ? l : 0u;            // padding bits stay zero
                p |= l << (i * B);
            }
            const uint32_t lowpart = p << sh;
            const uint32_t highpart = sh ? (p >> (32u - sh)) : 0u;      // zero unless the 8 B bits cross a word
            uint32_t mine = 0u;
#pragma unroll
            for (int k = 0; k < B; ++k) {
                uint32_t c = ((wi == (uint32_t)k) ? lowpart : 0u) | ((wi + 1u == (uint32_t)k) ? highpart : 0u);
                c |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
                c |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
                if (t == (uint32_t)k) mine = c;
            }
            if (t < (uint32_t)B && g * B + t < wpr) out_words[g * B + t] = mine;
            if (DW) {
                if (full) {
#pragma unroll
                    for (int q = 0; q < 2; ++q)
                        *(float4 *)(dWr + j0 + 4 * q) = make_float4(dq[4 * q], dq[4 * q + 1], dq[4 * q + 2], dq[4 * q + 3]);
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (j0 + i < m) dWr[j0 + i] = dq[i];
                }
            }
        }
    }
}

template <int B>
__device__ __forceinline__ void pack_row_dispatch(PackRound &cur, const float *Wr, const float *alpha, uint32_t m, bool vec_ok,
                                                  const float *thr, const int *thl, const float *cbf, uint32_t *ow,
                                                  uint32_t wpr, float *dWr) {
    if (alpha) {
        if (dWr) pack_row_body<B, true, true>(cur, Wr, alpha, m, vec_ok, thr, thl, cbf, ow, wpr, dWr);
        else pack_row_body<B, true, false>(cur, Wr, alpha, m, vec_ok, thr, thl, cbf, ow, wpr, dWr);
    } else {
        if (dWr) pack_row_body<B, false, true>(cur, Wr, alpha, m, vec_ok, thr, thl, cbf, ow, wpr, dWr);
        else pack_row_body<B, false, false>(cur, Wr, alpha, m, vec_ok, thr, thl, cbf, ow, wpr, dWr);
    }
}

__global__ void __launch_bounds__(PACK_THREADS) pack_rows_kernel(const float *W, const float *alpha, long long m,
                                                                 long long ld, const uint8_t *bits,
                                                                 const double *cent, const float *upper,
                                                                 const int *rowpos, const PackPlan *plan,
                                                                 uint32_t *codes, uint16_t *codebooks, float *dW) {
    __shared__ __align__(16) float thr[16];
    __shared__ int thl[16];
    __shared__ float cbf[16];
    const long long row = blockIdx.x;
    const int tid = threadIdx.x;
    // the first round of weights is on its way while the row's bounds are put in order
    const float *Wr = W + row * ld;
    float *dWr = dW ? dW + row * m : nullptr;
    const bool vec_ok = ((((uintptr_t)Wr) | (uintptr_t)alpha | (uintptr_t)dWr) & 15) == 0;
    PackRound first;
    if (alpha) pack_load_round<true>(first, Wr, alpha, (uint32_t)m, (uint32_t)tid >> 2, vec_ok);
    else pack_load_round<false>(first, Wr, alpha, (uint32_t)m, (uint32_t)tid >> 2, vec_ok);

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
    uint32_t *ow = codes + word0;
    switch (b) {
        case 1: pack_row_dispatch<1>(first, Wr, alpha, (uint32_t)m, vec_ok, thr, thl, cbf, ow, (uint32_t)wpr, dWr); break;
        case 2: pack_row_dispatch<2>(first, Wr, alpha, (uint32_t)m, vec_ok, thr, thl, cbf, ow, (uint32_t)wpr, dWr); break;
        case 3: pack_row_dispatch<3>(first, Wr, alpha, (uint32_t)m, vec_ok, thr, thl, cbf, ow, (uint32_t)wpr, dWr); break;
        default: pack_row_dispatch<4>(first, Wr, alpha, (uint32_t)m, vec_ok, thr, thl, cbf, ow, (uint32_t)wpr, dWr); break;
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
