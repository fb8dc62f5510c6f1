// Exact solution of the bit allocation problem that Alg. 1 approximates: the knapsack form stated with the
// mixed-precision problem, unit cost per row and bit, solved by dynamic programming on the device.  It is the
// yardstick for the greedy allocation (how much error the greedy loop leaves on the table), not part of the
// quantisation path.
//
// f_i[x] = least error of rows 0..i-1 when they hold exactly x bits above bmin in total,
// f_{i+1}[x] = min_d f_i[x - d] + E[i][bmin + d]   (equal sums keep the smaller d).
// A workgroup keeps 4 consecutive states per thread in registers and walks DP_ROWS rows per launch; the
// d <= 3 states a thread needs from its left neighbour travel through LDS (one barrier per row).  Several
// workgroups tile the state axis with an overlap of 3 * DP_ROWS states on the left: whatever a workgroup
// cannot know about the states left of its span spoils 3 more states per row, which is exactly the overlap
// that the neighbouring workgroup owns.  The choices d are stored as bytes, n x (states rounded up to 8),
// and a last kernel walks them back from the best final state.
#include "skim_common.h"

#include <math.h>

namespace {

constexpr int DP_THREADS = 256;
constexpr int DP_SPT = 4;                              // states per thread
constexpr int DP_ROWS = 64;                            // rows per launch
constexpr int DP_MAXD = 3;                             // bmax - bmin at most
constexpr int DP_HALO = DP_MAXD * DP_ROWS;
constexpr int DP_SPAN = DP_THREADS * DP_SPT;           // states one workgroup holds
constexpr int DP_OUT = DP_SPAN - DP_HALO;              // states one workgroup owns (a multiple of 4)
constexpr int TR_THREADS = 1024;

constexpr int TR_ROWS = 64;                            // rows the trace-back stages at a time
constexpr int TR_WIN = 256;                            // >= DP_MAXD * TR_ROWS + 1 states

__global__ void dp_init_kernel(double *__restrict__ f, long long nstates) {
    const long long x = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (x < nstates) f[x] = x == 0 ? 0.0 : INFINITY;
}

__global__ void __launch_bounds__(DP_THREADS) dp_rows_kernel(const double *__restrict__ E, int nb, long long i0,
                                                            int nrows, long long X, long long xs,
                                                            const double *__restrict__ fin, double *__restrict__ fout,
                                                            uint8_t *__restrict__ choice) {
    __shared__ double hal[2][DP_THREADS][DP_MAXD];
    const int t = threadIdx.x;
    const long long out_lo = (long long)blockIdx.x * DP_OUT;
    const long long s0 = out_lo - DP_HALO + (long long)t * DP_SPT;   // first state of this thread
    double f[DP_SPT];
#pragma unroll
    for (int e = 0; e < DP_SPT; ++e) {
        const long long x = s0 + e;
        f[e] = (x >= 0 && x <= X) ? fin[x] : INFINITY;
    }
    const bool owns = s0 >= out_lo && s0 < xs;
    for (int r = 0; r < nrows; ++r) {
        const int buf = r & 1;
#pragma unroll
        for (int k = 0; k < DP_MAXD; ++k) hal[buf][t][k] = f[DP_SPT - DP_MAXD + k];
        __syncthreads();
        double ext[DP_MAXD + DP_SPT];
#pragma unroll
        for (int k = 0; k < DP_MAXD; ++k) ext[k] = t > 0 ? hal[buf][t - 1][k] : INFINITY;
#pragma unroll
        for (int e = 0; e < DP_SPT; ++e) ext[DP_MAXD + e] = f[e];
        const double *Ei = E + (i0 + r) * nb;
        double ed[DP_MAXD + 1];
#pragma unroll
        for (int d = 0; d <= DP_MAXD; ++d) ed[d] = d < nb ? Ei[d] : INFINITY;
        unsigned packed = 0;
#pragma unroll
        for (int e = 0; e < DP_SPT; ++e) {
            double best = ext[DP_MAXD + e] + ed[0];
            unsigned arg = 0;
#pragma unroll
            for (int d = 1; d <= DP_MAXD; ++d) {
                const double c = ext[DP_MAXD + e - d] + ed[d];
                if (c < best) { best = c; arg = d; }
            }
            f[e] = best;
            packed |= arg << (8 * e);
        }
        if (owns) *(unsigned *)(choice + (i0 + r) * xs + s0) = packed;
    }
    if (s0 >= out_lo) {
#pragma unroll
        for (int e = 0; e < DP_SPT; ++e)
            if (s0 + e <= X) fout[s0 + e] = f[e];
    }
}

// Smallest state that attains the least final error, then the walk back through the choices: 64 rows of a
// 256-state window are staged in LDS at a time (the state falls by at most 3 per row), so that the
// dependent reads of the walk hit LDS instead of HBM.
__global__ void __launch_bounds__(TR_THREADS) dp_trace_kernel(const double *__restrict__ f, long long X, long long xs,
                                                             const uint8_t *__restrict__ choice, long long n, int bmin,
                                                             long long budget, uint8_t *__restrict__ bits,
                                                             double *__restrict__ info) {
    __shared__ double wbest[TR_THREADS / 64];
    __shared__ long long warg[TR_THREADS / 64];
    __shared__ long long sh_x;
    __shared__ uint8_t win[TR_ROWS][TR_WIN];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    double best = INFINITY;
    long long arg = 0x7fffffffffffffffll;
    for (long long x = t; x <= X; x += TR_THREADS) {
        const double v = f[x];
        if (v < best) { best = v; arg = x; }   // x ascending per thread: the first minimum stays
    }
    for (int o = 32; o >= 1; o >>= 1) {
        const double ob = __shfl_xor(best, o, 64);
        const long long oa = __shfl_xor(arg, o, 64);
        if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    }
    if (lane == 0) { wbest[wave] = best; warg[wave] = arg; }
    __syncthreads();
    if (t == 0) {
        for (int w = 1; w < TR_THREADS / 64; ++w)
            if (wbest[w] < best || (wbest[w] == best && warg[w] < arg)) { best = wbest[w]; arg = warg[w]; }
        sh_x = arg;
        info[0] = best;
        info[1] = (double)(n * bmin + arg);
        info[2] = (double)budget;
    }
    __syncthreads();
    for (long long hi = n; hi > 0; hi -= TR_ROWS) {
        const long long lo = hi > TR_ROWS ? hi - TR_ROWS : 0;       // rows lo..hi-1, walked downwards
        const long long x = sh_x;
        const long long w0 = x - (TR_WIN - 1);                      // window = states w0..x
        for (int idx = t; idx < TR_ROWS * TR_WIN; idx += TR_THREADS) {
            const int r = idx / TR_WIN, c = idx % TR_WIN;
            const long long row = lo + r, st = w0 + c;
            win[r][c] = (row < hi && st >= 0) ? choice[row * xs + st] : 0;
        }
        __syncthreads();
        if (t == 0) {
            long long cx = x;
            for (long long row = hi - 1; row >= lo; --row) {
                int d = win[row - lo][cx - w0];
                if (d > cx) d = (int)cx;                            // only a table with non-finite entries gets here
                bits[row] = (uint8_t)(bmin + d);
                cx -= d;
            }
            sh_x = cx;
        }
        __syncthreads();
    }
}

bool dp_sizes(int64_t n, int bmin, int bmax, double avg_bits, int64_t *B, int64_t *X, int64_t *xs) {
    if (n < 1 || n > (1ll << 24) || bmin < 1 || bmax < bmin || bmax - bmin > DP_MAXD || bmax > 7) return false;
    *B = (int64_t)floor(avg_bits * (double)n + 1e-9);
    if (*B < (int64_t)bmin * n || *B > (int64_t)bmax * n) return false;
    *X = *B - (int64_t)bmin * n;
    *xs = (*X + 1 + 7) & ~(int64_t)7;
    return true;
}

}  // namespace

extern "C" size_t skim_dp_allocate_scratch_bytes(int64_t n, int bmin, int bmax, double avg_bits) {
    int64_t B, X, xs;
    if (!dp_sizes(n, bmin, bmax, avg_bits, &B, &X, &xs)) return 0;
    return (size_t)2 * xs * sizeof(double) + (size_t)n * xs + 512;
}

extern "C" skim_status skim_dp_allocate(skim_ctx *ctx, const double *E, int64_t n, int bmin, int bmax, double avg_bits,
                                        uint8_t *bits, double *info, void *scratch, size_t scratch_bytes) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!E || !bits || !info || !scratch) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_dp_allocate: NULL argument");
    if (n < 1 || n > (1ll << 24)) SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "skim_dp_allocate: n = %lld out of range", (long long)n);
    if (bmin < 1 || bmax < bmin || bmax > 7 || bmax - bmin > DP_MAXD)
        SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_dp_allocate: bit range [%d,%d] (at most %d apart, within 1..7)", bmin, bmax, DP_MAXD);
    int64_t B, X, xs;
    if (!dp_sizes(n, bmin, bmax, avg_bits, &B, &X, &xs))
        SKIM_FAIL(ctx, SKIM_ERR_BUDGET, "budget outside [%lld, %lld]", (long long)(bmin * n), (long long)(bmax * n));
    const size_t need = skim_dp_allocate_scratch_bytes(n, bmin, bmax, avg_bits);
    if (scratch_bytes < need)
        SKIM_FAIL(ctx, SKIM_ERR_WORKSPACE, "skim_dp_allocate: scratch of %zu bytes, %zu needed", scratch_bytes, need);
    if (((uintptr_t)scratch & 255) != 0) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_dp_allocate: scratch not 256-byte aligned");
    double *fa = (double *)scratch, *fb = fa + xs;
    uint8_t *choice = (uint8_t *)(fb + xs);
    const int nb = bmax - bmin + 1;
    hipLaunchKernelGGL(dp_init_kernel, dim3((unsigned)((xs + 255) / 256)), dim3(256), 0, ctx->stream, fa, (long long)xs);
    const unsigned grid = (unsigned)((X + 1 + DP_OUT - 1) / DP_OUT);
    for (int64_t i0 = 0; i0 < n; i0 += DP_ROWS) {
        const int nrows = (int)(n - i0 < DP_ROWS ? n - i0 : DP_ROWS);
        hipLaunchKernelGGL(dp_rows_kernel, dim3(grid), dim3(DP_THREADS), 0, ctx->stream, E, nb, (long long)i0, nrows,
                           (long long)X, (long long)xs, (const double *)fa, fb, choice);
        double *tmp = fa; fa = fb; fb = tmp;
    }
    hipLaunchKernelGGL(dp_trace_kernel, dim3(1), dim3(TR_THREADS), 0, ctx->stream, (const double *)fa, (long long)X,
                       (long long)xs, (const uint8_t *)choice, (long long)n, bmin, (long long)B, bits, info);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}
