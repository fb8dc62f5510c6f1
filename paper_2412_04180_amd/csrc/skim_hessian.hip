// Layer-wise Hessian proxy from calibration activations (Sec. 3.4: H ~ X X^T in the paper's
// column convention; here X is N x m row-major, one activation vector per row, so
// H = X^T X / N, m x m).  bf16 inputs, bf16 MFMA (v_mfma_f32_32x32x16_bf16) with float32
// accumulation over chunks of 2048 activations, the chunks added up in float64.
#include "skim_common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int HT = 128;            // output tile (rows and columns of H = columns of X)
constexpr int HK = 64;             // activations per LDS tile
constexpr int HK_PAD = HK + 8;     // bf16 per LDS row: 144 bytes (16-byte aligned; operand reads and staging
                                   // stores of a 16-lane group fall into distinct banks)
constexpr int H_THREADS = 256;
constexpr int FLUSH_TILES = 32;    // float32 accumulators are added into float64 every 32 tiles = 2048 activations

// LDS tile T[c][k]: column c of the X tile, HK consecutive activations (k contiguous: one
// ds_read_b128 gives a lane its 8 bf16 of an MFMA operand).
struct XTile {
    uint16_t t[HT][HK_PAD];
};
constexpr size_t H_LDS_BYTES = 4 * sizeof(XTile);     // two operands, double-buffered

// Half of the workgroup stages each operand tile.  One thread moves 8 activations x 8 neighbouring columns:
// eight 16-byte loads (a wavefront covers 8 activation rows x 128 contiguous bytes per instruction), an
// 8 x 8 transpose of 16-bit values in registers, eight 16-byte LDS stores (one per column).
struct Staged {
    uint32_t r[8][4];
};
__device__ __forceinline__ void load_task(const uint16_t *__restrict__ X, long long N, long long m, long long k0,
                                          long long c0, int st, bool vec, Staged &s) {
    const int ab = st & 7, cg = st >> 3;             // 8-activation block, 8-column group
    const long long c = c0 + 8 * cg;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const long long k = k0 + 8 * ab + t;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (k < N) {
            const uint16_t *src = X + k * m + c;
            if (vec && c + 8 <= m) {
                v = *(const uint4 *)src;             // m % 8 == 0 and X 16-byte aligned
            } else {
                uint32_t e[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) e[q] = (c + q < m) ? src[q] : 0u;
                v = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
            }
        }
        s.r[t][0] = v.x; s.r[t][1] = v.y; s.r[t][2] = v.z; s.r[t][3] = v.w;
    }
}
__device__ __forceinline__ void store_task(XTile &T, int st, const Staged &s) {
    const int ab = st & 7, cg = st >> 3;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        uint32_t o[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t a = s.r[2 * d][c >> 1], b = s.r[2 * d + 1][c >> 1];
            o[d] = (c & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
        }
        *(uint4 *)&T.t[8 * cg + c][8 * ab] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

__global__ void __launch_bounds__(H_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) xtx_kernel(const uint16_t *__restrict__ X, long long N, long long m,
                                                        float *__restrict__ H, int vec) {
    extern __shared__ __align__(16) unsigned char smem[];
    XTile *TI = (XTile *)smem, *TJ = TI + 2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;
    const long long i0 = (long long)blockIdx.y * HT, j0 = (long long)blockIdx.x * HT;
    // threads 0..127 stage the tile of columns i0.., threads 128..255 the tile of columns j0..
    const int st = tid & 127;
    const bool stage_j = tid >= 128;
    const long long sc0 = stage_j ? j0 : i0;
    XTile *const ST = stage_j ? TJ : TI;

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
    Staged sg;
    load_task(X, N, m, 0, sc0, st, vec != 0, sg);
    store_task(ST[0], st, sg);
    __syncthreads();
    for (long long kt = 0; kt < ntile; ++kt) {
        const int buf = (int)(kt & 1);
        if (kt + 1 < ntile) load_task(X, N, m, (kt + 1) * HK, sc0, st, vec != 0, sg);
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
        if (kt + 1 < ntile) store_task(ST[buf ^ 1], st, sg);
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
    if (!ctx->xtx_lds_enabled) {
        SKIM_HIP(ctx, hipFuncSetAttribute((const void *)xtx_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)H_LDS_BYTES));
        ctx->xtx_lds_enabled = 1;
    }
    const unsigned nt = (unsigned)((m + HT - 1) / HT);
    const int vec = (m % 8 == 0) && (((uintptr_t)X_bf16 & 15) == 0);     // rows of X start 16-byte aligned
    hipLaunchKernelGGL(xtx_kernel, dim3(nt, nt), dim3(H_THREADS), H_LDS_BYTES, ctx->stream, X_bf16, (long long)N,
                       (long long)m, H, vec);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}
