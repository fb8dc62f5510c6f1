// Layer-wise Hessian proxy from calibration activations (Sec. 3.4: H ~ X X^T in the paper's
// column convention; here X is N x m row-major, one activation vector per row, so
// H = X^T X / N, m x m).  bf16 inputs, bf16 MFMA (v_mfma_f32_32x32x16_bf16) with float32
// accumulation over chunks of 512 activations, the chunks added up in float64.
#include "skim_common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int HT = 128;            // output tile (rows and columns of H = columns of X)
constexpr int HK = 32;             // activations per LDS tile
constexpr int HK_PAD = HK + 8;     // bf16 per LDS row: 80 bytes, keeps 16-byte alignment
constexpr int H_THREADS = 256;
constexpr int FLUSH_TILES = 16;    // float32 accumulators are added into float64 every 16 tiles = 512 activations

// LDS tile T[c][k]: column c of the X tile, HK consecutive activations (k contiguous: one
// ds_read_b128 gives a lane its 8 bf16 of an MFMA operand).
struct XTile {
    uint16_t t[HT][HK_PAD];
};

// One thread moves 8 activations x 2 neighbouring columns: 8 coalesced 4-byte loads, two 16-byte LDS stores.
struct Staged {
    uint32_t r[8];
};
__device__ __forceinline__ void load_task(const uint16_t *__restrict__ X, long long N, long long m, long long k0,
                                          long long c0, int tid, Staged &s) {
    const int kb = tid >> 6, cp = tid & 63;          // 8-activation block, column pair
    const long long c = c0 + 2 * cp;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const long long k = k0 + 8 * kb + t;
        uint32_t v = 0;
        if (k < N) {
            const uint16_t *src = X + k * m + c;
            if (c + 1 < m) v = *(const uint32_t *)src;       // m even and c even: 4-byte aligned
            else if (c < m) v = src[0];
        }
        s.r[t] = v;
    }
}
__device__ __forceinline__ void store_task(XTile &T, int tid, const Staged &s) {
    const int kb = tid >> 6, cp = tid & 63;
    uint32_t lo[4], hi[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        lo[t] = (s.r[2 * t] & 0xffffu) | (s.r[2 * t + 1] << 16);
        hi[t] = (s.r[2 * t] >> 16) | (s.r[2 * t + 1] & 0xffff0000u);
    }
    *(uint4 *)&T.t[2 * cp][8 * kb] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    *(uint4 *)&T.t[2 * cp + 1][8 * kb] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
}

__global__ void __launch_bounds__(H_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) xtx_kernel(const uint16_t *__restrict__ X, long long N, long long m,
                                                        float *__restrict__ H) {
    __shared__ __align__(16) XTile TI[2], TJ[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;
    const long long i0 = (long long)blockIdx.y * HT, j0 = (long long)blockIdx.x * HT;

    floatx16 acc[2][2];
    double acc64[2][2][16];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                acc[a][b][e] = 0.f;
                acc64[a][b][e] = 0.0;
            }

    const long long ntile = (N + HK - 1) / HK;
    Staged si, sj;
    load_task(X, N, m, 0, i0, tid, si);
    load_task(X, N, m, 0, j0, tid, sj);
    store_task(TI[0], tid, si);
    store_task(TJ[0], tid, sj);
    __syncthreads();
    for (long long kt = 0; kt < ntile; ++kt) {
        const int buf = (int)(kt & 1);
        if (kt + 1 < ntile) {
            load_task(X, N, m, (kt + 1) * HK, i0, tid, si);
            load_task(X, N, m, (kt + 1) * HK, j0, tid, sj);
        }
#pragma unroll
        for (int ks = 0; ks < HK / 16; ++ks) {
            // operand of a lane: 8 consecutive activations 16 ks + 8 (lane / 32) .. + 7 of one column
            const int kk = 16 * ks + 8 * lhi;
            const bf16x8 a0 = *(const bf16x8 *)&TI[buf].t[wr * 64 + l32][kk];
            const bf16x8 a1 = *(const bf16x8 *)&TI[buf].t[wr * 64 + 32 + l32][kk];
            const bf16x8 b0 = *(const bf16x8 *)&TJ[buf].t[wc * 64 + l32][kk];
            const bf16x8 b1 = *(const bf16x8 *)&TJ[buf].t[wc * 64 + 32 + l32][kk];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
        }
        if ((kt % FLUSH_TILES) == FLUSH_TILES - 1 || kt + 1 == ntile) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        acc64[a][b][e] += (double)acc[a][b][e];
                        acc[a][b][e] = 0.f;
                    }
        }
        if (kt + 1 < ntile) {
            store_task(TI[buf ^ 1], tid, si);
            store_task(TJ[buf ^ 1], tid, sj);
        }
        __syncthreads();
    }

    // accumulator element e of a 32 x 32 tile: row = 8*(e/4) + 4*(lane/32) + e%4, column = lane%32
    const double inv = 1.0 / (double)N;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const long long i = i0 + wr * 64 + a * 32 + 8 * (e >> 2) + 4 * lhi + (e & 3);
                const long long j = j0 + wc * 64 + b * 32 + l32;
                if (i < m && j < m) H[i * m + j] = (float)(acc64[a][b][e] * inv);
            }
}

}  // namespace

extern "C" skim_status skim_hessian_from_activations(skim_ctx *ctx, const uint16_t *X_bf16, int64_t N, int64_t m,
                                                     float *H) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!X_bf16 || !H) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_hessian_from_activations: NULL argument");
    if (N < 1 || m < 2 || (m & 1) || m > 0x7fffffff || ((uintptr_t)X_bf16 & 3))
        SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "skim_hessian_from_activations: need N >= 1, m even, X 4-byte aligned (N=%lld m=%lld)",
                  (long long)N, (long long)m);
    const unsigned nt = (unsigned)((m + HT - 1) / HT);
    hipLaunchKernelGGL(xtx_kernel, dim3(nt, nt), dim3(H_THREADS), 0, ctx->stream, X_bf16, (long long)N, (long long)m, H);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}
