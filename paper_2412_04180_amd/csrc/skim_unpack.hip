// Readers of the packed model (Sec. 4.2 last paragraph and App. D.2: rows of equal bit width
// are gathered and processed together; Sec. 5.4: binary16 codebooks): dequantisation to a
// dense matrix and the matrix-vector product that looks every weight up in its row's
// codebook.  Both walk the layout skim_pack writes: rows by (bits, row index), a b-bit row =
// ceil(m*b/32) little-endian words, column j at bit j*b.
#include "skim_common.h"

#include <hip/hip_fp16.h>

namespace {

constexpr int UNPACK_THREADS = 256;

struct RowPlace {        // where packed row p lives
    int b;               // its bit width
    long long word0;     // first code word
    long long cb0;       // first codebook entry
};

// group_word_offset[b] .. [b+1] holds the b-bit rows, each ceil(m*b/32) words.
__device__ __forceinline__ RowPlace place_row(const long long *gwo, long long m, long long p) {
    RowPlace r{0, 0, 0};
    long long rows_before = 0, cb = 0;
    for (int b = 1; b <= 4; ++b) {
        const long long wpr = (m * b + 31) / 32;
        const long long rows = (gwo[b + 1] - gwo[b]) / wpr;
        if (p < rows_before + rows) {
            r.b = b;
            r.word0 = gwo[b] + (p - rows_before) * wpr;
            r.cb0 = cb + (p - rows_before) * (1ll << b);
            return r;
        }
        rows_before += rows;
        cb += rows * (1ll << b);
    }
    return r;   // b == 0: p is past the last row
}

// Column j of a B-bit row: bits [j*B, j*B + B) of the row's little-endian word stream.  Neighbouring
// threads take neighbouring columns, so the loads of x, alpha and the code words coalesce.
template <int B, bool MATVEC>
__device__ __forceinline__ void row_body(const uint32_t *__restrict__ row_words, long long m, const float *cbf,
                                         const float *__restrict__ alpha, const float *__restrict__ x,
                                         float *__restrict__ Wq_row, double &acc) {
    const uint32_t mm = (uint32_t)m;   // m * 4 < 2^31 * 32 is checked on the host: bit offsets fit 32 bits for m < 2^29
#pragma unroll 4
    for (uint32_t j = threadIdx.x; j < mm; j += UNPACK_THREADS) {
        const uint32_t bit = j * B;
        const uint32_t wi = bit >> 5;
        const int sh = (int)(bit & 31);
        uint32_t v = row_words[wi] >> sh;
        if ((32 % B) != 0 && sh + B > 32) v |= row_words[wi + 1] << (32 - sh);   // only 3-bit codes straddle words
        const float c = cbf[v & ((1u << B) - 1u)];
        const float q = alpha ? __fmul_rn(alpha[j], c) : c;   // the dequantised weight, float32
        if (MATVEC) acc = fma((double)q, (double)x[j], acc);
        else Wq_row[j] = q;
    }
}

template <bool MATVEC>
__global__ void __launch_bounds__(UNPACK_THREADS) packed_rows_kernel(const uint32_t *codes, const long long *gwo,
                                                                    const int *row_perm, const uint16_t *codebooks,
                                                                    const float *alpha, long long m, const float *x,
                                                                    double *y, float *Wq) {
    __shared__ float cbf[16];
    __shared__ double red[UNPACK_THREADS / 64];
    const long long p = blockIdx.x;
    const RowPlace pl = place_row(gwo, m, p);
    if (pl.b == 0) return;
    const int tid = threadIdx.x;
    if (tid < (1 << pl.b)) cbf[tid] = __half2float(__ushort_as_half(codebooks[pl.cb0 + tid]));
    __syncthreads();
    const long long row = row_perm[p];
    const uint32_t *rw = codes + pl.word0;
    float *Wq_row = MATVEC ? nullptr : Wq + row * m;
    double acc = 0.0;
    switch (pl.b) {
        case 1: row_body<1, MATVEC>(rw, m, cbf, alpha, x, Wq_row, acc); break;
        case 2: row_body<2, MATVEC>(rw, m, cbf, alpha, x, Wq_row, acc); break;
        case 3: row_body<3, MATVEC>(rw, m, cbf, alpha, x, Wq_row, acc); break;
        default: row_body<4, MATVEC>(rw, m, cbf, alpha, x, Wq_row, acc); break;
    }
    if (MATVEC) {
        for (int d = 32; d >= 1; d >>= 1) acc += __shfl_down(acc, d, 64);
        if ((tid & 63) == 0) red[tid >> 6] = acc;
        __syncthreads();
        if (tid == 0) {
            double s = 0.0;
            for (int w2 = 0; w2 < UNPACK_THREADS / 64; ++w2) s += red[w2];
            y[row] = s;
        }
    }
}

// The matrix-vector product proper: a workgroup takes MV_ROWS packed rows at once so that x and alpha are read
// once for all of them (one row per workgroup re-reads 8 bytes of x and alpha per weight from L2, far more
// than the 0.4 bytes of codes the weight costs in HBM).  A lane owns 32 consecutive columns = B whole code
// words of every row; all its loads of an iteration (8 + 8 float4 of x and alpha, MV_ROWS * B code words) are
// independent and in flight together.  Rows of different widths may share a workgroup (at the group borders).
constexpr int MV_THREADS = 256;
constexpr int MV_ROWS = 8;

template <int B>
__device__ __forceinline__ double mv_chunk(const uint32_t *__restrict__ rw, uint32_t w0, uint32_t wpr, const float *cbf,
                                           const float (&al)[32], const double (&xd)[32], bool scaled) {
    uint32_t wd[B + 1];
#pragma unroll
    for (int k = 0; k < B; ++k) wd[k] = (w0 + k < wpr) ? rw[w0 + k] : 0u;
    wd[B] = 0u;
    double acc = 0.0;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        constexpr uint32_t mask = (1u << B) - 1u;
        const int bit = e * B, wi = bit >> 5, sh = bit & 31;
        uint32_t v = wd[wi] >> sh;
        if (sh + B > 32) v |= wd[wi + 1] << (32 - sh);
        const float c = cbf[v & mask];
        const float q = scaled ? __fmul_rn(al[e], c) : c;
        acc = fma((double)q, xd[e], acc);
    }
    return acc;
}

__global__ void __launch_bounds__(MV_THREADS) matvec_rows_kernel(const uint32_t *codes, const long long *gwo,
                                                                const int *row_perm, const uint16_t *codebooks,
                                                                const float *alpha, long long n, long long m,
                                                                const float *x, double *y) {
    __shared__ float cbf[MV_ROWS][16];
    __shared__ double red[MV_ROWS][MV_THREADS / 64];
    __shared__ RowPlace places[MV_ROWS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long p0 = (long long)blockIdx.x * MV_ROWS;
    if (tid < MV_ROWS) {
        RowPlace pl{0, 0, 0};
        if (p0 + tid < n) pl = place_row(gwo, m, p0 + tid);
        places[tid] = pl;
    }
    __syncthreads();
    if (tid < MV_ROWS * 16) {
        const int r = tid >> 4, k = tid & 15;
        const RowPlace pl = places[r];
        cbf[r][k] = (pl.b > 0 && k < (1 << pl.b)) ? __half2float(__ushort_as_half(codebooks[pl.cb0 + k])) : 0.0f;
    }
    __syncthreads();
    double acc[MV_ROWS];
#pragma unroll
    for (int r = 0; r < MV_ROWS; ++r) acc[r] = 0.0;
    const uint32_t mm = (uint32_t)m;
    const uint32_t nchunk = (mm + 31) >> 5;
    for (uint32_t ch = tid; ch < nchunk; ch += MV_THREADS) {
        const uint32_t j0 = ch << 5;
        float al[32];
        double xd[32];
        if (j0 + 32 <= mm) {
            const float4 *x4 = (const float4 *)(x + j0);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float4 v = x4[k];
                xd[4 * k] = v.x; xd[4 * k + 1] = v.y; xd[4 * k + 2] = v.z; xd[4 * k + 3] = v.w;
            }
            if (alpha) {
                const float4 *a4 = (const float4 *)(alpha + j0);
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float4 v = a4[k];
                    al[4 * k] = v.x; al[4 * k + 1] = v.y; al[4 * k + 2] = v.z; al[4 * k + 3] = v.w;
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                const bool in = j0 + e < mm;
                xd[e] = in ? (double)x[j0 + e] : 0.0;     // columns past the row: code 0 times 0
                al[e] = (in && alpha) ? alpha[j0 + e] : 1.0f;
            }
        }
#pragma unroll
        for (int r = 0; r < MV_ROWS; ++r) {
            const RowPlace pl = places[r];
            const uint32_t *rw = codes + pl.word0;
            const uint32_t wpr = (uint32_t)((m * pl.b + 31) / 32);
            switch (pl.b) {
                case 1: acc[r] += mv_chunk<1>(rw, ch * 1u, wpr, cbf[r], al, xd, alpha != nullptr); break;
                case 2: acc[r] += mv_chunk<2>(rw, ch * 2u, wpr, cbf[r], al, xd, alpha != nullptr); break;
                case 3: acc[r] += mv_chunk<3>(rw, ch * 3u, wpr, cbf[r], al, xd, alpha != nullptr); break;
                case 4: acc[r] += mv_chunk<4>(rw, ch * 4u, wpr, cbf[r], al, xd, alpha != nullptr); break;
                default: break;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < MV_ROWS; ++r) {
        double a = acc[r];
        for (int d = 32; d >= 1; d >>= 1) a += __shfl_down(a, d, 64);
        if (lane == 0) red[r][wave] = a;
    }
    __syncthreads();
    if (tid < MV_ROWS && places[tid].b > 0) {
        double s2 = 0.0;
        for (int w2 = 0; w2 < MV_THREADS / 64; ++w2) s2 += red[tid][w2];
        y[row_perm[p0 + tid]] = s2;
    }
}

// The same product with float32 arithmetic, for a reader that is limited by the packed bytes it streams rather
// than by float64 issue: y_i = sum_j c_ij * (alpha_j x_j), c_ij = f32(codebook_i[code_ij]), fused multiply-adds in
// float32.  A workgroup takes MVF_ROWS rows; a lane owns 32 consecutive columns = B whole code words of every
// row and forms alpha_j x_j once for all rows.  Per weight: one shift, one mask (the code, already scaled to a
// byte offset), one LDS read of the codebook entry (row base in the instruction's offset field), one FMA.
constexpr int MVF_THREADS = 256;
constexpr int MVF_ROWS = 8;

// the 32 weights of one row whose B code words are in wd[0..B) (wd[B] = 0)
template <int B, int R>
__device__ __forceinline__ float mvf_words(const uint32_t (&wd)[B + 1], const float (*cbf)[16], const float (&xs)[32]) {
    float acc0 = 0.0f, acc1 = 0.0f;
    const char *base = (const char *)cbf[R];
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        constexpr uint32_t mask4 = ((1u << B) - 1u) << 2;       // the code times 4: byte offset of a float
        const int bit = e * B, wi = bit >> 5, sh = bit & 31;
        // (code << 2) = bits [sh, sh + B) of the stream moved to bits [2, 2 + B)
        uint32_t v = sh >= 2 ? (wd[wi] >> (sh - 2)) : (wd[wi] << (2 - sh));
        if (sh + B > 32) v |= wd[wi + 1] << (34 - sh);
        const float c = *(const float *)(base + (v & mask4));
        if (e & 1) acc1 = fmaf(c, xs[e], acc1);
        else acc0 = fmaf(c, xs[e], acc0);
    }
    return acc0 + acc1;
}

template <int B, int R>
__device__ __forceinline__ float mvf_chunk(const uint32_t *__restrict__ rw, uint32_t w0, uint32_t wpr,
                                           const float (*cbf)[16], const float (&xs)[32]) {
    uint32_t wd[B + 1];
#pragma unroll
    for (int k = 0; k < B; ++k) wd[k] = (w0 + k < wpr) ? rw[w0 + k] : 0u;
    wd[B] = 0u;
    return mvf_words<B, R>(wd, cbf, xs);
}

// All MVF_ROWS rows of the workgroup have B bits (rows are packed by bit width, so this is every workgroup but
// the few that straddle two groups): the code words of all rows are requested before the first is used.
template <int B, int R>
__device__ __forceinline__ void mvf_same_rows(const uint32_t (&wd)[MVF_ROWS][B + 1], const float (*cbf)[16],
                                              const float (&xs)[32], float (&acc)[MVF_ROWS]) {
    if constexpr (R < MVF_ROWS) {
        acc[R] += mvf_words<B, R>(wd[R], cbf, xs);
        mvf_same_rows<B, R + 1>(wd, cbf, xs, acc);
    }
}
template <int B>
__device__ __forceinline__ void mvf_same(const uint32_t *codes, const RowPlace *places, long long m, uint32_t ch,
                                         const float (*cbf)[16], const float (&xs)[32], float (&acc)[MVF_ROWS]) {
    const uint32_t wpr = (uint32_t)((m * B + 31) / 32);
    uint32_t wd[MVF_ROWS][B + 1];
#pragma unroll
    for (int r = 0; r < MVF_ROWS; ++r) {
        const uint32_t *rw = codes + places[r].word0;
#pragma unroll
        for (int k = 0; k < B; ++k) wd[r][k] = (ch * B + k < wpr) ? rw[ch * B + k] : 0u;
        wd[r][B] = 0u;
    }
    mvf_same_rows<B, 0>(wd, cbf, xs, acc);
}

template <int R>
__device__ __forceinline__ void mvf_rows(const uint32_t *codes, const RowPlace *places, long long m, uint32_t ch,
                                         const float (*cbf)[16], const float (&xs)[32], float (&acc)[MVF_ROWS]) {
    if constexpr (R < MVF_ROWS) {
        const RowPlace pl = places[R];
        const uint32_t *rw = codes + pl.word0;
        const uint32_t wpr = (uint32_t)((m * pl.b + 31) / 32);
        switch (pl.b) {
            case 1: acc[R] += mvf_chunk<1, R>(rw, ch * 1u, wpr, cbf, xs); break;
            case 2: acc[R] += mvf_chunk<2, R>(rw, ch * 2u, wpr, cbf, xs); break;
            case 3: acc[R] += mvf_chunk<3, R>(rw, ch * 3u, wpr, cbf, xs); break;
            case 4: acc[R] += mvf_chunk<4, R>(rw, ch * 4u, wpr, cbf, xs); break;
            default: break;
        }
        mvf_rows<R + 1>(codes, places, m, ch, cbf, xs, acc);
    }
}

template <bool ALIGNED>
__global__ void __launch_bounds__(MVF_THREADS) matvec_f32_kernel(const uint32_t *codes, const long long *gwo,
                                                                 const int *row_perm, const uint16_t *codebooks,
                                                                 const float *alpha, long long n, long long m,
                                                                 const float *x, float *y) {
    __shared__ float cbf[MVF_ROWS][16];
    __shared__ float red[MVF_ROWS][MVF_THREADS / 64];
    __shared__ RowPlace places[MVF_ROWS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long p0 = (long long)blockIdx.x * MVF_ROWS;
    if (tid < MVF_ROWS) {
        RowPlace pl{0, 0, 0};
        if (p0 + tid < n) pl = place_row(gwo, m, p0 + tid);
        places[tid] = pl;
    }
    __syncthreads();
    if (tid < MVF_ROWS * 16) {
        const int r = tid >> 4, k = tid & 15;
        const RowPlace pl = places[r];
        cbf[r][k] = (pl.b > 0 && k < (1 << pl.b)) ? __half2float(__ushort_as_half(codebooks[pl.cb0 + k])) : 0.0f;
    }
    __syncthreads();
    float acc[MVF_ROWS];
#pragma unroll
    for (int r = 0; r < MVF_ROWS; ++r) acc[r] = 0.0f;
    // the bit width all rows of this workgroup share, 0 when they differ (or some are past the end)
    int same_b = places[0].b;
#pragma unroll
    for (int r = 1; r < MVF_ROWS; ++r) same_b = (places[r].b == same_b) ? same_b : 0;
    same_b = __builtin_amdgcn_readfirstlane(same_b);
    const uint32_t mm = (uint32_t)m;
    const uint32_t nchunk = (mm + 31) >> 5;
    for (uint32_t ch = tid; ch < nchunk; ch += MVF_THREADS) {
        const uint32_t j0 = ch << 5;
        float xs[32];                                  // alpha_j * x_j (columns past the row: 0)
        if (ALIGNED && j0 + 32 <= mm) {
            const float4 *x4 = (const float4 *)(x + j0);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float4 v = x4[k];
                xs[4 * k] = v.x; xs[4 * k + 1] = v.y; xs[4 * k + 2] = v.z; xs[4 * k + 3] = v.w;
            }
            if (alpha) {
                const float4 *a4 = (const float4 *)(alpha + j0);
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float4 v = a4[k];
                    xs[4 * k] *= v.x; xs[4 * k + 1] *= v.y; xs[4 * k + 2] *= v.z; xs[4 * k + 3] *= v.w;
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                const bool in = j0 + e < mm;
                xs[e] = in ? (alpha ? alpha[j0 + e] * x[j0 + e] : x[j0 + e]) : 0.0f;
            }
        }
        switch (same_b) {
            case 1: mvf_same<1>(codes, places, m, ch, cbf, xs, acc); break;
            case 2: mvf_same<2>(codes, places, m, ch, cbf, xs, acc); break;
            case 3: mvf_same<3>(codes, places, m, ch, cbf, xs, acc); break;
            case 4: mvf_same<4>(codes, places, m, ch, cbf, xs, acc); break;
            default: mvf_rows<0>(codes, places, m, ch, cbf, xs, acc); break;
        }
    }
#pragma unroll
    for (int r = 0; r < MVF_ROWS; ++r) {
        float a = acc[r];
        for (int d = 32; d >= 1; d >>= 1) a += __shfl_down(a, d, 64);
        if (lane == 0) red[r][wave] = a;
    }
    __syncthreads();
    if (tid < MVF_ROWS && places[tid].b > 0) {
        float s2 = 0.0f;
        for (int w2 = 0; w2 < MVF_THREADS / 64; ++w2) s2 += red[tid][w2];
        y[row_perm[p0 + tid]] = s2;
    }
}

skim_status check_packed(skim_ctx *ctx, const void *codes, const void *gwo, const void *perm, const void *cbs, int64_t n,
                         int64_t m, const char *who) {
    if (!codes || !gwo || !perm || !cbs) SKIM_FAIL(ctx, SKIM_ERR_ARG, "%s: NULL argument", who);
    if (n < 1 || n > 0x7fffffff || m < 1 || m >= (1ll << 29))
        SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "%s: bad shape n=%lld m=%lld", who, (long long)n, (long long)m);
    return SKIM_OK;
}

}  // namespace

extern "C" skim_status skim_unpack(skim_ctx *ctx, const uint32_t *codes, const int64_t *group_word_offset,
                                   const int32_t *row_perm, const uint16_t *codebooks_fp16, const float *alpha,
                                   int64_t n, int64_t m, float *Wq) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if ((st = check_packed(ctx, codes, group_word_offset, row_perm, codebooks_fp16, n, m, "skim_unpack")) != SKIM_OK) return st;
    if (!Wq) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_unpack: Wq must not be NULL");
    hipLaunchKernelGGL(packed_rows_kernel<false>, dim3((unsigned)n), dim3(UNPACK_THREADS), 0, ctx->stream, codes,
                       (const long long *)group_word_offset, row_perm, codebooks_fp16, alpha, (long long)m,
                       (const float *)nullptr, (double *)nullptr, Wq);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}

extern "C" skim_status skim_dequant_matvec(skim_ctx *ctx, const uint32_t *codes, const int64_t *group_word_offset,
                                           const int32_t *row_perm, const uint16_t *codebooks_fp16, const float *alpha,
                                           int64_t n, int64_t m, const float *x, double *y) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if ((st = check_packed(ctx, codes, group_word_offset, row_perm, codebooks_fp16, n, m, "skim_dequant_matvec")) != SKIM_OK)
        return st;
    if (!x || !y) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_dequant_matvec: x and y must not be NULL");
    if ((((uintptr_t)x | (uintptr_t)alpha) & 15) == 0)
        hipLaunchKernelGGL(matvec_rows_kernel, dim3((unsigned)((n + MV_ROWS - 1) / MV_ROWS)), dim3(MV_THREADS), 0,
                           ctx->stream, codes, (const long long *)group_word_offset, row_perm, codebooks_fp16, alpha,
                           (long long)n, (long long)m, x, y);
    else   // x or alpha not aligned for 16-byte loads: one row per workgroup, 4-byte loads
        hipLaunchKernelGGL(packed_rows_kernel<true>, dim3((unsigned)n), dim3(UNPACK_THREADS), 0, ctx->stream, codes,
                           (const long long *)group_word_offset, row_perm, codebooks_fp16, alpha, (long long)m, x, y,
                           (float *)nullptr);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}

extern "C" skim_status skim_dequant_matvec_f32(skim_ctx *ctx, const uint32_t *codes, const int64_t *group_word_offset,
                                               const int32_t *row_perm, const uint16_t *codebooks_fp16,
                                               const float *alpha, int64_t n, int64_t m, const float *x, float *y) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if ((st = check_packed(ctx, codes, group_word_offset, row_perm, codebooks_fp16, n, m, "skim_dequant_matvec_f32")) != SKIM_OK)
        return st;
    if (!x || !y) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_dequant_matvec_f32: x and y must not be NULL");
    const dim3 grid((unsigned)((n + MVF_ROWS - 1) / MVF_ROWS));
    if ((((uintptr_t)x | (uintptr_t)alpha) & 15) == 0)
        hipLaunchKernelGGL(matvec_f32_kernel<true>, grid, dim3(MVF_THREADS), 0, ctx->stream, codes,
                           (const long long *)group_word_offset, row_perm, codebooks_fp16, alpha, (long long)n,
                           (long long)m, x, y);
    else
        hipLaunchKernelGGL(matvec_f32_kernel<false>, grid, dim3(MVF_THREADS), 0, ctx->stream, codes,
                           (const long long *)group_word_offset, row_perm, codebooks_fp16, alpha, (long long)n,
                           (long long)m, x, y);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}
