// Greedy mixed-precision bit allocation (Alg. 1, unit costs) on the device, so that the
// path error table -> allocation -> pack needs no round trip to the host.
//
// Same order as the host function: upgrade j of a row is taken when the running minimum
// k_j = min(g_1 .. g_j) of the row's reductions comes up, and the greedy loop takes the
// upgrades in the order (k descending, row ascending, j ascending).  The first T = budget -
// n * bmin of them are found by a most-significant-digit radix selection on the keys
// (8 digits of 8 bits, one workgroup), ties at the threshold value in index order.
#include "skim_common.h"

#include <math.h>

namespace {

constexpr int GA_THREADS = 1024;
constexpr size_t GA_LDS_KEYS = 128 * 1024;      // keys kept in LDS up to this many bytes (16384 keys)
typedef unsigned long long u64;

// float64 -> uint64 whose unsigned order is the order of the doubles (-0 folded into +0).
__device__ __forceinline__ u64 ordered_key(double x) {
    if (x == 0.0) x = 0.0;
    const u64 u = (u64)__double_as_longlong(x);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

// hist[dig] += 1 for the lanes with `valid`.  The lanes that share the digit of the first valid lane are
// counted with one atomic (the high digits of the keys are nearly constant; one atomic per key would
// serialise on a single LDS address); the others add on their own.
__device__ __forceinline__ void hist_add(unsigned *hist, bool valid, unsigned dig) {
    const u64 act = __ballot(valid);
    if (act == 0) return;
    const int leader = __ffsll((long long)act) - 1;
    const unsigned first = (unsigned)__builtin_amdgcn_readlane((int)dig, leader);   // leader is the same in every lane
    const u64 same = __ballot(valid && dig == first);
    if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[first], (unsigned)__popcll(same));
    else if (valid && dig != first) atomicAdd(&hist[dig], 1u);
}

__global__ void __launch_bounds__(GA_THREADS) greedy_select_kernel(const double *__restrict__ E, long long n, int bmin,
                                                                  int nb, long long T, u64 *keys_global,
                                                                  uint8_t *__restrict__ bits, long long *__restrict__ info,
                                                                  long long budget, int keys_in_lds) {
    // the keys are written, re-read for the ties, marked and read again for the bits: in LDS when they fit
    // (one workgroup: every trip to global memory is pure latency), else in the caller's workspace
    extern __shared__ __align__(16) unsigned char ga_smem[];
    u64 *keys = keys_in_lds ? (u64 *)ga_smem : keys_global;
    __shared__ unsigned hist[256];
    __shared__ u64 sh_prefix;
    __shared__ long long sh_rank;
    __shared__ int sh_single;
    __shared__ long long wsum[GA_THREADS / 64];
    __shared__ long long cnt[8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nu = nb - 1;
    const long long nk = n * nu;

    // keys: running minima of the reductions, row by row
    for (long long i = tid; i < n; i += GA_THREADS) {
        double k = 0.0;
        for (int j = 0; j < nu; ++j) {
            const double g = E[i * nb + j] - E[i * nb + j + 1];
            k = (j == 0 || g < k) ? g : k;
            keys[i * nu + j] = ordered_key(k);
        }
    }
    if (tid < 8) cnt[tid] = 0;
    __syncthreads();

    // up to 16 keys per thread stay in registers over the eight passes (tables of up to 5461 rows
    // at three upgrades per row); larger tables re-read the keys from global memory
    constexpr int KPT = 16;
    const bool in_regs = nk <= (long long)GA_THREADS * KPT;
    u64 rk[KPT];
    if (in_regs) {
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const long long q = tid + (long long)k * GA_THREADS;
            rk[k] = (q < nk) ? keys[q] : 0ull;
        }
    }

    // threshold = the T-th largest key (T >= 1): fix its digits from the top
    u64 prefix = 0;
    long long rank = T;            // rank among the keys that share the prefix fixed so far
    u64 thr = 0;
    long long R = 0;               // keys equal to the threshold that are still taken
    bool lone = false;             // exactly one key equals the threshold and it is taken: taken <=> key >= thr
    if (T > 0 && T < nk) {
        for (int d = 7; d >= 0; --d) {
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            const u64 hi_mask = (d == 7) ? 0ull : (~0ull << (8 * (d + 1)));
            if (in_regs) {
#pragma unroll
                for (int k = 0; k < KPT; ++k) {
                    const long long q = tid + (long long)k * GA_THREADS;
                    hist_add(hist, q < nk && (rk[k] & hi_mask) == prefix, (unsigned)(rk[k] >> (8 * d)) & 255u);
                }
            } else {
                for (long long q = tid; q < nk; q += GA_THREADS) {
                    const u64 key = keys[q];
                    hist_add(hist, (key & hi_mask) == prefix, (unsigned)(key >> (8 * d)) & 255u);
                }
            }
            __syncthreads();
            if (wave == 0) {
                // the bin that holds the rank-th largest key: lane l owns bins 4l .. 4l+3; suffix sums over the lanes
                const unsigned h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
                const long long mine = (long long)h0 + h1 + h2 + h3;
                long long inc = mine;                       // sum over lanes >= this one
                for (int dd = 1; dd < 64; dd <<= 1) {
                    const long long u = __shfl_down(inc, dd, 64);
                    if (lane + dd < 64) inc += u;
                }
                const long long above = inc - mine;         // keys in higher bins than this lane's
                if (above < rank && rank <= inc) {          // exactly one lane
                    long long r = rank - above;
                    int bin = 4 * lane + 3;
                    if ((long long)h3 < r) { r -= h3; bin = 4 * lane + 2;
                        if ((long long)h2 < r) { r -= h2; bin = 4 * lane + 1;
                            if ((long long)h1 < r) { r -= h1; bin = 4 * lane; } } }
                    sh_prefix = prefix | ((u64)bin << (8 * d));
                    sh_rank = r;
                    sh_single = (hist[bin] == 1u) ? 1 : 0;   // one key left under the new prefix: it is the threshold
                }
            }
            __syncthreads();
            prefix = sh_prefix;
            rank = sh_rank;
            const bool single = sh_single != 0;
            if (single && d > 0) {
                // the remaining digits are those of that key: its owner publishes it
                __syncthreads();   // every thread has read sh_prefix / sh_single before it is overwritten
                const u64 lo_mask = ~0ull << (8 * d);
                if (in_regs) {
#pragma unroll
                    for (int k = 0; k < KPT; ++k) {
                        const long long q = tid + (long long)k * GA_THREADS;
                        if (q < nk && (rk[k] & lo_mask) == prefix) sh_prefix = rk[k];
                    }
                } else {
                    for (long long q = tid; q < nk; q += GA_THREADS) {
                        const u64 key = keys[q];
                        if ((key & lo_mask) == prefix) sh_prefix = key;
                    }
                }
                __syncthreads();
                prefix = sh_prefix;
                lone = true;
                break;             // rank == 1 here
            }
        }
        thr = prefix;
        R = rank;                  // the first R keys equal to thr, in index order, are taken
    }

    // keys equal to the threshold: positions in index order (contiguous index ranges per thread)
    const long long per = (nk + GA_THREADS - 1) / GA_THREADS;
    const long long q0 = min(nk, per * tid), q1 = min(nk, q0 + per);
    long long eq_before = 0;
    if (T > 0 && T < nk && !lone) {
        long long mine = 0;
        for (long long q = q0; q < q1; ++q) mine += (keys[q] == thr) ? 1 : 0;
        long long inc = mine;
        for (int dd = 1; dd < 64; dd <<= 1) {
            const long long u = __shfl_up(inc, dd, 64);
            if (lane >= dd) inc += u;
        }
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        long long before = 0;
        for (int w2 = 0; w2 < wave; ++w2) before += wsum[w2];
        eq_before = before + inc - mine;
    }
    __syncthreads();
    // taken: key > thr, or key == thr among the first R equal ones; T >= nk takes everything.
    // Mark by overwriting the key with 1 / 0 (each thread owns its index range).  With a lone key at the threshold
    // the comparison key >= thr says it all and the rows are counted from the keys themselves.
    for (long long q = q0; q < q1 && !lone; ++q) {
        const u64 key = keys[q];
        bool take;
        if (T <= 0) take = false;
        else if (T >= nk) take = true;
        else if (key > thr) take = true;
        else if (key == thr) take = (eq_before++ < R);
        else take = false;
        keys[q] = take ? 1ull : 0ull;
    }
    __syncthreads();
    // rows per bit width: counted per wavefront with ballots (one LDS atomic per wavefront and width instead of
    // one per row on a handful of addresses)
    long long wcnt[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (long long i0 = 0; i0 < n; i0 += GA_THREADS) {
        const long long i = i0 + tid;
        int b = -1;
        if (i < n) {
            b = bmin;
            for (int j = 0; j < nu; ++j) {
                const u64 key = keys[i * nu + j];
                b += lone ? (key >= thr ? 1 : 0) : (int)key;
            }
            bits[i] = (uint8_t)b;
        }
#pragma unroll
        for (int v = 0; v < 8; ++v) wcnt[v] += __popcll(__ballot(b == v));
    }
    if (lane == 0) {
#pragma unroll
        for (int v = 0; v < 8; ++v)
            if (wcnt[v]) atomicAdd((unsigned long long *)&cnt[v], (unsigned long long)wcnt[v]);
    }
    __syncthreads();
    if (tid < 8) info[tid] = cnt[tid];
    if (tid == 0) {
        long long spent = 0;
        for (int b = 0; b < 8; ++b) spent += cnt[b] * b;
        info[8] = spent;
        info[9] = budget;
    }
}

}  // namespace

extern "C" skim_status skim_greedy_allocate_device(skim_ctx *ctx, const double *E, int64_t n, int bmin, int bmax,
                                                   double avg_bits, uint8_t *bits, int64_t *info) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!E || !bits || !info) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_greedy_allocate_device: NULL argument");
    if (n < 1 || n > (1ll << 24)) SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "skim_greedy_allocate_device: n = %lld out of range", (long long)n);
    if (bmin < 1 || bmax < bmin || bmax > 7) SKIM_FAIL(ctx, SKIM_ERR_ARG, "bit range [%d,%d] outside 1..7", bmin, bmax);
    const int64_t B = (int64_t)floor(avg_bits * (double)n + 1e-9);
    if (B < (int64_t)bmin * n || B > (int64_t)bmax * n)
        SKIM_FAIL(ctx, SKIM_ERR_BUDGET, "budget %lld outside [%lld, %lld]", (long long)B, (long long)(bmin * n), (long long)(bmax * n));
    const int nb = bmax - bmin + 1;
    const size_t need = (size_t)n * (nb > 1 ? nb - 1 : 1) * sizeof(u64);
    if (!ctx->ws || ctx->ws_bytes < need)
        SKIM_FAIL(ctx, SKIM_ERR_WORKSPACE, "workspace missing or smaller than skim_workspace_bytes(n, m)");
    const size_t key_bytes = (size_t)n * (nb > 1 ? nb - 1 : 1) * sizeof(u64);
    const int keys_in_lds = key_bytes <= GA_LDS_KEYS;
    if (keys_in_lds && !ctx->greedy_lds_enabled) {
        SKIM_HIP(ctx, hipFuncSetAttribute((const void *)greedy_select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)GA_LDS_KEYS));
        ctx->greedy_lds_enabled = 1;
    }
    hipLaunchKernelGGL(greedy_select_kernel, dim3(1), dim3(GA_THREADS), keys_in_lds ? key_bytes : 0, ctx->stream, E,
                       (long long)n, bmin, nb, (long long)(B - (int64_t)bmin * n), (u64 *)ctx->ws, bits, (long long *)info,
                       (long long)B, keys_in_lds);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}
