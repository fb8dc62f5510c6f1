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
    hipLaunchKernelGGL(packed_rows_kernel<true>, dim3((unsigned)n), dim3(UNPACK_THREADS), 0, ctx->stream, codes,
                       (const long long *)group_word_offset, row_perm, codebooks_fp16, alpha, (long long)m, x, y,
                       (float *)nullptr);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}
