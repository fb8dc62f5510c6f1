// Scaling-vector step of SKIM (Sec. 4.3, Alg. 2 inner loop; Alg. 3, training loop)
// for gfx950: centroids from fixed labels, the layer-wise (L-full, Sec. 3.4)
// loss tr(dW H dW^T), its gradient with respect to alpha and the Adam update.
//
//   c_ik  = sum_{j in k} s~_ij w~_ij / sum_{j in k} s~_ij      (calc_centroids(W*alpha^-1, L))
//   dW_ij = w_ij - alpha_j c_{i,L_ij}                           (W - replace(c, L) * alpha)
//   P     = dW H            matrix cores, float32 accumulation (the path's one dense contraction): bf16 MFMA on
//                           three-piece splits of the float32 operands (dwh_gemm3_kernel), or fp32 MFMA (dwh_gemm_kernel)
//   loss  = sum_ij P_ij dW_ij                                   float64 reduction
//   dloss/dalpha_l = -2 sum_i [ P_il c_{i,L_il}
//                    + Q_{i,L_il} s_il (w_il - 2 alpha_l c_{i,L_il}) / D_{i,L_il} ],
//   Q_ik = sum_{j in k} P_ij alpha_j,  D_ik = sum_{j in k} s~_ij  (gradient through the centroids).
#include "skim_common.h"

#include <math.h>

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Pieces of a float32 value for the contraction on the bf16 matrix cores (see dwh_gemm3_kernel)
__device__ __forceinline__ uint32_t bf16_rn(float f) {      // finite f
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float bf16_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ void split3(float x, uint32_t &p1, uint32_t &p2, uint32_t &p3) {
    p1 = bf16_rn(x);
    float r = x - bf16_f32(p1);       // exact
    p2 = bf16_rn(r);
    r -= bf16_f32(p2);                // exact; at most 8 significant bits are left
    p3 = bf16_rn(r);
}
__device__ __forceinline__ size_t plane_index(long long row, long long rows, long long k) {
    return ((size_t)(k >> 5) * (size_t)rows + (size_t)row) * 96 + (size_t)(k & 31);     // piece p at + 32 p
}


constexpr int PREP_THREADS = 256;
constexpr int BM = 128, BN = 128, BK = 16;
constexpr int A_STRIDE = BM + 4;   // k-major A tile, padded against bank conflicts of the transposing store
constexpr int GEMM_THREADS = 256;
constexpr int STRIP = 8;           // rows per workgroup in the gradient kernel

__device__ __forceinline__ double block_sum_256(double x, double *scratch /* >= 4 doubles */) {
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_down(x, d, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) scratch[wave] = x;
    __syncthreads();
    return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

// Per-cluster sums of a row with fixed labels: every wavefront adds into bins of its own in LDS (float64
// atomic adds), four copies per wavefront picked by the lane so that lanes with the same label seldom meet
// on one address; the copies are then added in a fixed order.
constexpr int BIN_COPIES = 4;
constexpr int BIN_SETS = (PREP_THREADS / 64) * BIN_COPIES;

__device__ __forceinline__ double bin_total(const double (*bins)[16], int k) {
    double t = 0.0;
#pragma unroll
    for (int b = 0; b < BIN_SETS; ++b) t += bins[b][k];
    return t;
}

// Per row: weighted cluster sums with fixed labels -> centroids c (n x 16 float64),
// masses Den (n x 16 float64), and the row of dW (float32, or its three bfloat16 pieces when dWp is given).
// kept (optional): per row, at kept + row * kept_stride, the centroid a cluster keeps when its members carry no
// sensitivity mass (what the clustering that produced the labels left there); without it such a centroid is 0.
__global__ void __launch_bounds__(PREP_THREADS) row_prep_kernel(const float *W, const float *S, const float *alpha,
                                                                long long m, long long ld, const uint8_t *labels,
                                                                double *cent, double *Den, float *dW, uint16_t *dWp,
                                                                const double *kept, long long kept_stride, int kept_n,
                                                                bool vec4) {
    __shared__ double binD[BIN_SETS][16], binN[BIN_SETS][16];
    __shared__ double csh[16];
    const long long row = blockIdx.x, nrows = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *Wr = W + row * ld, *Sr = S + row * ld;
    const uint8_t *Lr = labels + row * m;
    static_assert(BIN_SETS * 16 == PREP_THREADS, "one bin per thread to clear");
    (&binD[0][0])[tid] = 0.0;
    (&binN[0][0])[tid] = 0.0;
    __syncthreads();
    double *myD = binD[wave * BIN_COPIES + (lane & (BIN_COPIES - 1))];
    double *myN = binN[wave * BIN_COPIES + (lane & (BIN_COPIES - 1))];
    auto add_element = [&](float wt, float st, float a, int l) {
        if (alpha) {
            wt = __fdiv_rn(wt, a);
            st = __fmul_rn(__fmul_rn(st, a), a);
        }
        atomicAdd(&myD[l], (double)st);
        atomicAdd(&myN[l], (double)st * (double)wt);
    };
    // vec4: rows start 16-byte aligned (labels 4-byte) and m is a multiple of 4: four neighbouring columns per
    // thread and step, a quarter of the load instructions
    if (vec4) {
        for (long long j = 4ll * tid; j < m; j += 4 * PREP_THREADS) {
            const float4 w4 = *(const float4 *)(Wr + j), s4 = *(const float4 *)(Sr + j);
            const float4 a4 = alpha ? *(const float4 *)(alpha + j) : make_float4(1.f, 1.f, 1.f, 1.f);
            const uint32_t l4 = *(const uint32_t *)(Lr + j);
            add_element(w4.x, s4.x, a4.x, (int)(l4 & 15u));
            add_element(w4.y, s4.y, a4.y, (int)((l4 >> 8) & 15u));
            add_element(w4.z, s4.z, a4.z, (int)((l4 >> 16) & 15u));
            add_element(w4.w, s4.w, a4.w, (int)((l4 >> 24) & 15u));
        }
    } else {
        for (long long j = tid; j < m; j += PREP_THREADS) add_element(Wr[j], Sr[j], alpha ? alpha[j] : 1.0f, Lr[j] & 15);
    }
    __syncthreads();
    if (tid < 16) {
        const double d = bin_total(binD, tid), nn = bin_total(binN, tid);
        const double c = d > 0.0 ? nn / d : ((kept && tid < kept_n) ? kept[row * kept_stride + tid] : 0.0);
        csh[tid] = c;
        cent[row * 16 + tid] = c;
        Den[row * 16 + tid] = d;
    }
    __syncthreads();
    // dW as float32 for dwh_gemm_kernel, or as three bfloat16 pieces per value for dwh_gemm3_kernel
    if (vec4 && dWp) {
        for (long long j = 4ll * tid; j < m; j += 4 * PREP_THREADS) {
            const float4 w4 = *(const float4 *)(Wr + j);
            const float4 a4 = alpha ? *(const float4 *)(alpha + j) : make_float4(1.f, 1.f, 1.f, 1.f);
            const uint32_t l4 = *(const uint32_t *)(Lr + j);
            const float wv[4] = {w4.x, w4.y, w4.z, w4.w}, av[4] = {a4.x, a4.y, a4.z, a4.w};
            uint32_t pc[3][4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float d = (float)((double)wv[e] - (double)av[e] * csh[(l4 >> (8 * e)) & 15u]);
                split3(d, pc[0][e], pc[1][e], pc[2][e]);
            }
            uint16_t *o = dWp + plane_index(row, nrows, j);   // four neighbouring k stay inside one block of 32
#pragma unroll
            for (int q = 0; q < 3; ++q)
                *(uint2 *)(o + 32 * q) = make_uint2(pc[q][0] | (pc[q][1] << 16), pc[q][2] | (pc[q][3] << 16));
        }
        return;
    }
    for (long long j = tid; j < m; j += PREP_THREADS) {
        const double a = alpha ? (double)alpha[j] : 1.0;
        const float d = (float)((double)Wr[j] - a * csh[Lr[j] & 15]);
        if (dWp) {
            uint32_t p1, p2, p3;
            split3(d, p1, p2, p3);
            uint16_t *o = dWp + plane_index(row, nrows, j);
            o[0] = (uint16_t)p1;
            o[32] = (uint16_t)p2;
            o[64] = (uint16_t)p3;
        } else {
            dW[row * m + j] = d;
        }
    }
}

// P = dW * H on fp32 MFMA (v_mfma_f32_32x32x2_f32), 128 x 128 output tile per
// workgroup, four wavefronts in a 2 x 2 arrangement of 64 x 64 sub-tiles.  Four workgroups
// per compute unit (register budget 128 per lane): the 1024 tiles of a 4096 x 4096 layer are
// then resident at once instead of leaving a quarter of them for a thin second round.
// Epilogue: optional store of P and, per output row, sum_j P_ij dW_ij over the
// tile's columns in float64 -> partial[tile_col][row].
template <bool STORE_P>
__global__ void __launch_bounds__(GEMM_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) dwh_gemm_kernel(const float *__restrict__ A, const float *__restrict__ H,
                                                                int n, int m, float *__restrict__ P,
                                                                double *__restrict__ partial) {
    __shared__ float As[2][BK][A_STRIDE];
    __shared__ float Bs[2][BK][BN];
    __shared__ double rsum[2][BM];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int row0 = blockIdx.y * BM, col0 = blockIdx.x * BN;
    const int l32 = lane & 31, lhi = lane >> 5;

    // global -> register staging: A tile 128 x 16 (two float4 per thread), B tile 16 x 128 (two float4)
    const int a_r = tid >> 2, a_k = (tid & 3) * 4;     // rows a_r and a_r + 64
    const int b_k = tid >> 5, b_c = (tid & 31) * 4;    // k rows b_k and b_k + 8
    float4 ra[2], rb[2];
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = row0 + a_r + 64 * i;
            ra[i] = (r < n) ? *(const float4 *)(A + (long long)r * m + k0 + a_k) : make_float4(0.f, 0.f, 0.f, 0.f);
            const int c = col0 + b_c;
            const float *src = H + (long long)(k0 + b_k + 8 * i) * m + c;
            if (c + 3 < m) {
                rb[i] = *(const float4 *)src;
            } else {
                rb[i].x = (c + 0 < m) ? src[0] : 0.f;
                rb[i].y = (c + 1 < m) ? src[1] : 0.f;
                rb[i].z = (c + 2 < m) ? src[2] : 0.f;
                rb[i].w = 0.f;
            }
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = a_r + 64 * i;
            As[buf][a_k + 0][r] = ra[i].x;
            As[buf][a_k + 1][r] = ra[i].y;
            As[buf][a_k + 2][r] = ra[i].z;
            As[buf][a_k + 3][r] = ra[i].w;
            *(float4 *)&Bs[buf][b_k + 8 * i][b_c] = rb[i];
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int nk = m / BK;
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_tiles((kt + 1) * BK);
#pragma unroll
        for (int kp = 0; kp < BK / 2; ++kp) {
            const int k = 2 * kp + lhi;
            const float a0 = As[buf][k][wr * 64 + l32];
            const float a1 = As[buf][k][wr * 64 + 32 + l32];
            const float b0 = Bs[buf][k][wc * 64 + l32];
            const float b1 = Bs[buf][k][wc * 64 + 32 + l32];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
        if (kt + 1 < nk) store_tiles(buf ^ 1);
        __syncthreads();
    }

    // epilogue.  Accumulator element e of a 32 x 32 tile: row = 8*(e/4) + 4*(lane/32) + e%4, column = lane%32.
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int rl = wr * 64 + i * 32 + 8 * (e >> 2) + 4 * lhi + (e & 3);
            const int r = row0 + rl;
            double t = 0.0;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int c = col0 + wc * 64 + j * 32 + l32;
                if (r < n && c < m) {
                    const float p = acc[i][j][e];
                    if (STORE_P) P[(long long)r * m + c] = p;
                    t += (double)p * (double)A[(long long)r * m + c];
                }
            }
            // sum over the 32 lanes that share this row
            for (int o = 16; o >= 1; o >>= 1) t += __shfl_xor(t, o, 64);
            if (l32 == 0) rsum[wc][rl] = t;
        }
    }
    __syncthreads();
    if (tid < BM && row0 + tid < n) partial[(long long)blockIdx.x * n + row0 + tid] = rsum[0][tid] + rsum[1][tid];
}

// ---- the same contraction on the bf16 matrix cores -----------------------------------------------------------
// A float32 value is the exact sum of three bfloat16 values (8 + 8 + 8 significant bits, each piece the rounding of
// what the pieces before it leave), so x y = sum over the nine products of pieces, each exact in float32.  The six
// products with piece indices i + j <= 4 carry everything down to 2^-24 of |x y| -- the size of float32's own
// rounding -- and v_mfma_f32_32x32x16_bf16 does one of them for 16 k in half the time v_mfma_f32_32x32x2_f32
// needs for 2 k: 6 x 32 clocks against 512 per 16 k.  Accumulation is float32 in the matrix core either way.
// Layout of a split matrix ("planes"): for every block of 32 k, row after row, [piece 1 (32) | piece 2 (32) |
// piece 3 (32)] as 192 contiguous bytes: the rows of a tile for one 32-k step are one contiguous region of memory
// (64 lanes of a load instruction read 1024 consecutive bytes; with the blocks of a row side by side instead, an
// instruction read 192 bytes of each of six rows and the kernel sat at the rate the memory system serves that).
// H (m x m float32, symmetric, m % 32 == 0) -> its planes, row j of the planes = row j of H = column j of H.
__global__ void __launch_bounds__(256) split_rows_kernel(const float *__restrict__ H, long long rows, long long m,
                                                         uint16_t *__restrict__ Hp) {
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;     // 8 consecutive k of one row
    const long long per_row = m >> 3;
    if (g >= rows * per_row) return;
    const long long j = g / per_row, k = (g - j * per_row) << 3;
    const float4 a = *(const float4 *)(H + j * m + k), b = *(const float4 *)(H + j * m + k + 4);
    const float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    uint32_t p[3][8];
#pragma unroll
    for (int e = 0; e < 8; ++e) split3(x[e], p[0][e], p[1][e], p[2][e]);
    uint16_t *dst = Hp + plane_index(j, rows, k);
#pragma unroll
    for (int q = 0; q < 3; ++q)
        *(uint4 *)(dst + 32 * q) = make_uint4(p[q][0] | (p[q][1] << 16), p[q][2] | (p[q][3] << 16), p[q][4] | (p[q][5] << 16),
                                              p[q][6] | (p[q][7] << 16));
}

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
constexpr int G3_BM = 256, G3_BN = 128, G3_BK = 32, G3_THREADS = 512;
constexpr int G3_PITCH = 104;                  // bfloat16 per LDS row: 3 pieces x 32 k + 8 of padding = 208 bytes
constexpr int G3_ROWS = G3_BM + G3_BN;         // the dW rows of the tile, then the H rows
constexpr int G3_CHUNKS = G3_ROWS * 12 / G3_THREADS;      // 16-byte pieces a thread stages per step: 9
constexpr size_t G3_LDS_BYTES = 2 * (size_t)G3_ROWS * G3_PITCH * sizeof(uint16_t);   // double-buffered: 159744

// P = dW H from the planes of dW (n rows) and of H (m rows; H symmetric: its row j stands in for its column j).
// 256 x 128 output tile, 8 wavefronts (two per SIMD) of 64 x 64; 32 k per step, LDS double-buffered, the next
// step's rows staged through registers while this step's MFMAs run.  Epilogue as in dwh_gemm_kernel, with dW
// put together again from its pieces (exactly).
template <bool STORE_P>
__global__ void __launch_bounds__(G3_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
dwh_gemm3_kernel(const uint16_t *__restrict__ Ap, const uint16_t *__restrict__ Hp, int n, int m, float *__restrict__ P,
                 double *__restrict__ partial) {
    extern __shared__ __align__(16) unsigned char g3_smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int row0 = blockIdx.y * G3_BM, col0 = blockIdx.x * G3_BN;

    // staging: piece c = tid + 512 q of the 384 x 12 pieces of a step; consecutive lanes read consecutive 16 bytes
    const uint16_t *src[G3_CHUNKS];
    uint32_t dst[G3_CHUNKS];          // byte offset inside one LDS buffer
    bool ok[G3_CHUNKS];
#pragma unroll
    for (int q = 0; q < G3_CHUNKS; ++q) {
        const int c = tid + G3_THREADS * q;
        const int trow = c / 12, part = c - 12 * trow;
        const bool isa = trow < G3_BM;
        const long long grow = isa ? (long long)row0 + trow : (long long)col0 + (trow - G3_BM);
        ok[q] = grow < (isa ? (long long)n : (long long)m);
        src[q] = (isa ? Ap : Hp) + (size_t)(ok[q] ? grow : 0) * 96 + 8 * part;
        dst[q] = (uint32_t)(trow * G3_PITCH + 8 * part) * 2u;
    }
    // (pieces 0 .. 3071 of a step are rows of dW, the rest rows of H: q < 6 is all dW, q = 6 .. 8 all H)
    static_assert(6 * G3_THREADS == G3_BM * 12, "the dW rows of a step end on a whole pass of the workgroup");
    const size_t step_a = (size_t)n * 96, step_h = (size_t)m * 96;      // from one 32-k block to the next
    uint4 sg[G3_CHUNKS];
    auto load_step = [&](int kt) {
#pragma unroll
        for (int q = 0; q < G3_CHUNKS; ++q) {
            const uint4 v = *(const uint4 *)(src[q] + (size_t)kt * (q < 6 ? step_a : step_h));
            sg[q] = ok[q] ? v : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    auto store_step = [&](int buf, int q0, int q1) {
        unsigned char *base = g3_smem + (size_t)buf * (G3_ROWS * G3_PITCH * 2);
#pragma unroll
        for (int q = 0; q < G3_CHUNKS; ++q)
            if (q >= q0 && q < q1) *(uint4 *)(base + dst[q]) = sg[q];
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int nk = m / G3_BK;
    load_step(0);
    store_step(0, 0, G3_CHUNKS);
    load_step(nk > 1 ? 1 : 0);
    __syncthreads();
    // operand of a lane: 8 consecutive k (16 ks + 8 (lane / 32) ..) of piece p of row (lane % 32) of a 32-row block
    const uint32_t a_off = (uint32_t)((wr * 64 + l32) * G3_PITCH + 8 * lhi) * 2u;
    const uint32_t b_off = (uint32_t)((G3_BM + wc * 64 + l32) * G3_PITCH + 8 * lhi) * 2u;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        const unsigned char *tb = g3_smem + (size_t)buf * (G3_ROWS * G3_PITCH * 2);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8_t a[3][2], b[3][2];
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int x = 0; x < 2; ++x) {
                    a[p][x] = *(const bf16x8_t *)(tb + a_off + (uint32_t)(32 * x * G3_PITCH + 32 * p + 16 * ks) * 2u);
                    b[p][x] = *(const bf16x8_t *)(tb + b_off + (uint32_t)(32 * x * G3_PITCH + 32 * p + 16 * ks) * 2u);
                }
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y) {
                    // smallest products first
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][x], b[1][y], acc[x][y], 0, 0, 0);
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][x], b[2][y], acc[x][y], 0, 0, 0);
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2][x], b[0][y], acc[x][y], 0, 0, 0);
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][x], b[1][y], acc[x][y], 0, 0, 0);
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][x], b[0][y], acc[x][y], 0, 0, 0);
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][x], b[0][y], acc[x][y], 0, 0, 0);
                }
        }
        // the next step's rows, requested a whole step ago, go to the other buffer (past the end: a repeat, never read)
        store_step(buf ^ 1, 0, G3_CHUNKS);
        load_step(min(kt + 2, nk - 1));
        __syncthreads();
    }

    // epilogue.  Accumulator element e of a 32 x 32 tile: row = 8*(e/4) + 4*(lane/32) + e%4, column = lane%32.
    double *rsum = (double *)g3_smem;          // [2][G3_BM]; the tiles are no longer read
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int rl = wr * 64 + i * 32 + 8 * (e >> 2) + 4 * lhi + (e & 3);
            const int r = row0 + rl;
            double t = 0.0;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int c = col0 + wc * 64 + j * 32 + l32;
                if (r < n && c < m) {
                    const float p = acc[i][j][e];
                    if (STORE_P) P[(long long)r * m + c] = p;
                    const uint16_t *ap = Ap + plane_index(r, n, c);
                    const float dw = (bf16_f32(ap[0]) + bf16_f32(ap[32])) + bf16_f32(ap[64]);     // exact
                    t += (double)p * (double)dw;
                }
            }
            // sum over the 32 lanes that share this row
            for (int o = 16; o >= 1; o >>= 1) t += __shfl_xor(t, o, 64);
            if (l32 == 0) rsum[wc * G3_BM + rl] = t;
        }
    }
    __syncthreads();
    if (tid < G3_BM && row0 + tid < n) partial[(long long)blockIdx.x * n + row0 + tid] = rsum[tid] + rsum[G3_BM + tid];
}

// row_loss[i] = sum over column tiles (one thread per row, neighbouring threads on neighbouring rows of every
// tile's partials; four running sums keep four loads in flight), left in partial[i] for the total.
__global__ void __launch_bounds__(256) loss_rows_kernel(double *partial, int ntile, long long n, double *row_loss,
                                                        long long row_stride) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    double r[4] = {0.0, 0.0, 0.0, 0.0};
    int t = 0;
    for (; t + 3 < ntile; t += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) r[u] += partial[(long long)(t + u) * n + i];
    }
    for (; t < ntile; ++t) r[t & 3] += partial[(long long)t * n + i];
    const double tot = (r[0] + r[1]) + (r[2] + r[3]);
    if (row_loss) row_loss[i * row_stride] = tot;
    partial[i] = tot;
}

// loss = sum_i partial[i] (single workgroup, fixed order).
__global__ void __launch_bounds__(1024) loss_total_kernel(const double *partial, long long n, double *loss) {
    __shared__ double sh[16];
    double acc = 0.0;
    for (long long i = threadIdx.x; i < n; i += 1024) acc += partial[i];
    for (int d = 32; d >= 1; d >>= 1) acc += __shfl_down(acc, d, 64);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int w = 0; w < 16; ++w) s += sh[w];
        *loss = s;
    }
}

static void launch_loss_finish(hipStream_t stream, double *partial, int ntile, long long n, double *loss, double *row_loss,
                               long long row_stride) {
    hipLaunchKernelGGL(loss_rows_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, partial, ntile, n,
                       row_loss, row_stride);
    hipLaunchKernelGGL(loss_total_kernel, dim3(1), dim3(1024), 0, stream, (const double *)partial, n, loss);
}

// Gradient terms.  One workgroup walks STRIP consecutive rows; per row it forms
// Q_ik = sum_{j in k} P_ij alpha_j (LDS bins as in row_prep_kernel), then adds each column's term to the
// thread's private column sums.  A thread owns the columns tid, tid + 256, ...: with REG (m <= 16 * 256)
// their sums, alpha and the row's P and labels stay in registers, so a row is read from HBM once;
// otherwise the sums live in gpart and the row is read twice.  gpart[strip][l] is reduced over the strips
// afterwards.
constexpr int GRAD_NC = 16;

template <bool REG>
__global__ void __launch_bounds__(PREP_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) grad_rows_kernel(const float *W, const float *S, const float *alpha,
                                                                 long long n, long long m, long long ld,
                                                                 const uint8_t *labels, const float *P,
                                                                 const double *cent, const double *Den,
                                                                 double *gpart, bool vec4) {
    __shared__ double binQ[BIN_SETS][16];
    __shared__ double rsh[16], csh[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long r0 = (long long)blockIdx.x * STRIP;
    double *gp = gpart + (long long)blockIdx.x * m;
    double gacc[GRAD_NC];
    float al[GRAD_NC];
    // The columns of a thread (REG): tid, tid + 256, ... -- or, when the rows can be read 16 bytes at a time (vec4),
    // four groups of four neighbouring columns 4 (tid + 256 q) .. + 3: a quarter of the load instructions, and a
    // row then arrives in a third of the time.
    auto colof = [&](int c) -> long long {
        return vec4 ? 4ll * (tid + (long long)(c >> 2) * PREP_THREADS) + (c & 3) : tid + (long long)c * PREP_THREADS;
    };
    if (REG) {
#pragma unroll
        for (int c = 0; c < GRAD_NC; ++c) {
            const long long l = colof(c);
            gacc[c] = 0.0;
            al[c] = l < m ? alpha[l] : 0.0f;
        }
    } else {
        for (long long l = tid; l < m; l += PREP_THREADS) gp[l] = 0.0;
    }
    double *myQ = binQ[wave * BIN_COPIES + (lane & (BIN_COPIES - 1))];
    for (long long row = r0; row < min(n, r0 + STRIP); ++row) {
        const float *Pr = P + row * m;
        const uint8_t *Lr = labels + row * m;
        const float *Wr = W + row * ld, *Sr = S + row * ld;
        (&binQ[0][0])[tid] = 0.0;
        // the row's cluster masses and centroids are requested now by the 16 threads that need them between the
        // barriers below, where every other thread waits for them
        double den_k = 0.0, cen_k = 0.0;
        if (tid < 16) {
            den_k = Den[row * 16 + tid];
            cen_k = cent[row * 16 + tid];
        }
        __syncthreads();      // bins cleared; the previous row's rsh/csh are no longer read
        float pv[GRAD_NC], wv[GRAD_NC], sv[GRAD_NC];
        int lv[GRAD_NC];
        if (REG) {
            if (vec4) {
#pragma unroll
                for (int q = 0; q < GRAD_NC / 4; ++q) {
                    const long long l = colof(4 * q);
                    float4 p4 = make_float4(0.f, 0.f, 0.f, 0.f), w4 = p4, s4 = p4;
                    uint32_t l4 = 0u;
                    if (l < m) {          // m is a multiple of 4 here: the four columns are inside together
                        p4 = *(const float4 *)(Pr + l);
                        w4 = *(const float4 *)(Wr + l);
                        s4 = *(const float4 *)(Sr + l);
                        l4 = *(const uint32_t *)(Lr + l);
                    }
                    pv[4 * q] = p4.x; pv[4 * q + 1] = p4.y; pv[4 * q + 2] = p4.z; pv[4 * q + 3] = p4.w;
                    wv[4 * q] = w4.x; wv[4 * q + 1] = w4.y; wv[4 * q + 2] = w4.z; wv[4 * q + 3] = w4.w;
                    sv[4 * q] = s4.x; sv[4 * q + 1] = s4.y; sv[4 * q + 2] = s4.z; sv[4 * q + 3] = s4.w;
                    lv[4 * q] = (int)(l4 & 15u); lv[4 * q + 1] = (int)((l4 >> 8) & 15u);
                    lv[4 * q + 2] = (int)((l4 >> 16) & 15u); lv[4 * q + 3] = (int)((l4 >> 24) & 15u);
                }
            } else {
#pragma unroll
                for (int c = 0; c < GRAD_NC; ++c) {
                    const long long l = colof(c);
                    const bool in = l < m;
                    pv[c] = in ? Pr[l] : 0.0f;
                    lv[c] = in ? (Lr[l] & 15) : 0;
                    wv[c] = in ? Wr[l] : 0.0f;
                    sv[c] = in ? Sr[l] : 0.0f;
                }
            }
#pragma unroll
            for (int c = 0; c < GRAD_NC; ++c)
                if (colof(c) < m) atomicAdd(&myQ[lv[c]], (double)pv[c] * (double)al[c]);
        } else {
            for (long long j = tid; j < m; j += PREP_THREADS)
                atomicAdd(&myQ[Lr[j] & 15], (double)Pr[j] * (double)alpha[j]);
        }
        __syncthreads();
        if (tid < 16) {
            const double q = bin_total(binQ, tid), d = den_k;
            rsh[tid] = d > 0.0 ? q / d : 0.0;
            csh[tid] = cen_k;
        }
        __syncthreads();
        if (REG) {
#pragma unroll
            for (int c = 0; c < GRAD_NC; ++c) {
                const double a = (double)al[c], cc = csh[lv[c]];
                const double term = (double)pv[c] * cc + rsh[lv[c]] * (double)sv[c] * ((double)wv[c] - 2.0 * a * cc);
                gacc[c] += -2.0 * term;
            }
        } else {
            for (long long l = tid; l < m; l += PREP_THREADS) {
                const int k = Lr[l] & 15;
                const double a = (double)alpha[l], cc = csh[k];
                const double term = (double)Pr[l] * cc + rsh[k] * (double)Sr[l] * ((double)Wr[l] - 2.0 * a * cc);
                gp[l] += -2.0 * term;   // the same thread owns column l for every row of the strip
            }
        }
    }
    if (REG) {
#pragma unroll
        for (int c = 0; c < GRAD_NC; ++c) {
            const long long l = colof(c);
            if (l < m) gp[l] = gacc[c];
        }
    }
}

// Column sums of the per-strip gradient terms, then the Adam update.  16 columns per workgroup (m / 16 workgroups:
// one per CU at 4096 columns); the strips are shared out to 64 groups of threads (a column's 64 partial sums are
// added in a fixed order).
constexpr int ADAM_COLS = 16, ADAM_GROUPS = 64;

__global__ void __launch_bounds__(ADAM_COLS * ADAM_GROUPS) adam_kernel(const double *gpart, int nstrip, long long m,
                                                                      float *alpha, float *am, float *av, float lr,
                                                                      float beta1, float beta2, float eps, float bc1,
                                                                      float bc2, float *grad_out) {
    __shared__ double part[ADAM_GROUPS][ADAM_COLS];
    const int c = threadIdx.x % ADAM_COLS, g = threadIdx.x / ADAM_COLS;
    const long long l = (long long)blockIdx.x * ADAM_COLS + c;
    double acc = 0.0;
    if (l < m)
        for (int st = g; st < nstrip; st += ADAM_GROUPS) acc += gpart[(long long)st * m + l];
    part[g][c] = acc;
    __syncthreads();
    if (g != 0 || l >= m) return;
    double g64 = 0.0;
#pragma unroll
    for (int k = 0; k < ADAM_GROUPS; ++k) g64 += part[k][c];
    const float gr = (float)g64;
    if (grad_out) grad_out[l] = gr;
    const float m1 = beta1 * am[l] + (1.0f - beta1) * gr;
    const float v1 = beta2 * av[l] + (1.0f - beta2) * gr * gr;
    am[l] = m1;
    av[l] = v1;
    const float mh = m1 / bc1, vh = v1 / bc2;
    alpha[l] = alpha[l] - lr * mh / (sqrtf(vh) + eps);
}

struct LossWs {
    float *dW, *P;
    uint16_t *dWp, *Hp;      // pieces of dW and of H for dwh_gemm3_kernel (null: the float32 kernel is used)
    double *cent, *Den, *partial, *gpart;
    int ntile, nstrip;
};

// The contraction runs on the bf16 matrix cores when the rows split into whole 32-k blocks and are long enough to
// fill a step pipeline; otherwise on the float32 ones.
bool use_pieces(int64_t m) { return (m % G3_BK) == 0 && m >= 128; }

skim_status carve(skim_ctx *ctx, int64_t n, int64_t m, bool need_grad, LossWs &w) {
    skim_ws_cursor cur{(char *)ctx->ws, 0, ctx->ws_bytes};
    w.ntile = (int)((m + BN - 1) / BN);
    w.nstrip = (int)((n + STRIP - 1) / STRIP);
    w.dW = nullptr;
    w.dWp = w.Hp = nullptr;
    if (use_pieces(m)) {        // (first in the workspace: skim_train_scale keeps the pieces of H across its steps)
        w.Hp = (uint16_t *)cur.take((size_t)m * m * 3 * sizeof(uint16_t));
        w.dWp = (uint16_t *)cur.take((size_t)n * m * 3 * sizeof(uint16_t));
    } else {
        w.dW = (float *)cur.take((size_t)n * m * sizeof(float));
    }
    w.cent = (double *)cur.take((size_t)n * 16 * sizeof(double));
    w.Den = (double *)cur.take((size_t)n * 16 * sizeof(double));
    w.partial = (double *)cur.take((size_t)w.ntile * n * sizeof(double));
    w.P = nullptr;
    w.gpart = nullptr;
    bool ok = (w.dW || (w.dWp && w.Hp)) && w.cent && w.Den && w.partial;
    if (need_grad) {
        w.P = (float *)cur.take((size_t)n * m * sizeof(float));
        w.gpart = (double *)cur.take((size_t)w.nstrip * m * sizeof(double));
        ok = ok && w.P && w.gpart;
    }
    if (!ok) SKIM_FAIL(ctx, SKIM_ERR_WORKSPACE, "workspace missing or smaller than skim_workspace_bytes(n, m)");
    return SKIM_OK;
}

// P = dW H (and the per-tile row sums of P o dW) by whichever kernel the workspace was carved for.  h_ready: the
// pieces of H are already in w.Hp (skim_train_scale splits H once per round of steps).
skim_status launch_contraction(skim_ctx *ctx, const LossWs &w, const float *H, int64_t n, int64_t m, bool store_p,
                               bool h_ready) {
    if (w.dWp) {
        if (!ctx->gemm3_lds_enabled) {
            SKIM_HIP(ctx, hipFuncSetAttribute((const void *)dwh_gemm3_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)G3_LDS_BYTES));
            SKIM_HIP(ctx, hipFuncSetAttribute((const void *)dwh_gemm3_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)G3_LDS_BYTES));
            ctx->gemm3_lds_enabled = 1;
        }
        if (!h_ready)
            hipLaunchKernelGGL(split_rows_kernel, dim3((unsigned)((m * (m / 8) + 255) / 256)), dim3(256), 0, ctx->stream, H,
                               (long long)m, (long long)m, w.Hp);
        const dim3 grid((unsigned)((m + G3_BN - 1) / G3_BN), (unsigned)((n + G3_BM - 1) / G3_BM));
        if (store_p)
            hipLaunchKernelGGL(dwh_gemm3_kernel<true>, grid, dim3(G3_THREADS), G3_LDS_BYTES, ctx->stream, w.dWp, w.Hp, (int)n,
                               (int)m, w.P, w.partial);
        else
            hipLaunchKernelGGL(dwh_gemm3_kernel<false>, grid, dim3(G3_THREADS), G3_LDS_BYTES, ctx->stream, w.dWp, w.Hp, (int)n,
                               (int)m, (float *)nullptr, w.partial);
    } else {
        const dim3 grid(w.ntile, (unsigned)((n + BM - 1) / BM));
        if (store_p)
            hipLaunchKernelGGL(dwh_gemm_kernel<true>, grid, dim3(GEMM_THREADS), 0, ctx->stream, w.dW, H, (int)n, (int)m, w.P,
                               w.partial);
        else
            hipLaunchKernelGGL(dwh_gemm_kernel<false>, grid, dim3(GEMM_THREADS), 0, ctx->stream, w.dW, H, (int)n, (int)m,
                               (float *)nullptr, w.partial);
    }
    return SKIM_OK;
}

// rows of W and S start 16-byte aligned, alpha is, and the labels of a row start 4-byte aligned (m is a multiple of 16)
bool rows_vec4(const float *W, const float *S, const float *alpha, const uint8_t *labels, int64_t ld) {
    return (ld % 4) == 0 && (((uintptr_t)W | (uintptr_t)S | (uintptr_t)alpha) & 15) == 0 && ((uintptr_t)labels & 3) == 0;
}

skim_status check_shape(skim_ctx *ctx, int64_t n, int64_t m, int64_t ld) {
    if (n < 1 || n > 0x7fffffff || m < BK || m > 0x7fffffff || ld < m || (m % BK) != 0)
        SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "layer loss needs n >= 1, m a multiple of %d, ld >= m (n=%lld m=%lld ld=%lld)", BK,
                  (long long)n, (long long)m, (long long)ld);
    return SKIM_OK;
}

}  // namespace

extern "C" skim_status skim_layer_loss(skim_ctx *ctx, const float *W, const float *S, const float *alpha,
                                       const float *H, int64_t n, int64_t m, int64_t ld, const uint8_t *labels,
                                       double *loss, double *row_loss) {
    return skim_layer_loss_strided(ctx, W, S, alpha, H, n, m, ld, labels, loss, row_loss, 1, nullptr, 0, 0);
}

skim_status skim_layer_loss_strided(skim_ctx *ctx, const float *W, const float *S, const float *alpha, const float *H,
                                    int64_t n, int64_t m, int64_t ld, const uint8_t *labels, double *loss,
                                    double *row_loss, int64_t row_stride, const double *kept, int64_t kept_stride,
                                    int kept_n) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!W || !S || !H || !labels || !loss) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_layer_loss: NULL argument");
    if ((st = check_shape(ctx, n, m, ld)) != SKIM_OK) return st;
    if ((uintptr_t)H & 15) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_layer_loss: H must be 16-byte aligned");
    LossWs w;
    if ((st = carve(ctx, n, m, false, w)) != SKIM_OK) return st;
    hipLaunchKernelGGL(row_prep_kernel, dim3((unsigned)n), dim3(PREP_THREADS), 0, ctx->stream, W, S, alpha, (long long)m,
                       (long long)ld, labels, w.cent, w.Den, w.dW, w.dWp, kept, (long long)kept_stride, kept_n,
                       rows_vec4(W, S, alpha, labels, ld));
    if ((st = launch_contraction(ctx, w, H, n, m, false, false)) != SKIM_OK) return st;
    launch_loss_finish(ctx->stream, w.partial, w.ntile, (long long)n, loss, row_loss, (long long)row_stride);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}

namespace {
skim_status scale_step_impl(skim_ctx *ctx, const float *W, const float *S, const float *H, int64_t n, int64_t m,
                            int64_t ld, const uint8_t *labels, float *alpha, float *adam_m, float *adam_v, int64_t t,
                            const skim_adam_opts *opts, double *loss_before, float *grad_out, bool h_ready);
}

extern "C" skim_status skim_scale_step(skim_ctx *ctx, const float *W, const float *S, const float *H, int64_t n,
                                       int64_t m, int64_t ld, const uint8_t *labels, float *alpha, float *adam_m,
                                       float *adam_v, int64_t t, const skim_adam_opts *opts, double *loss_before,
                                       float *grad_out) {
    return scale_step_impl(ctx, W, S, H, n, m, ld, labels, alpha, adam_m, adam_v, t, opts, loss_before, grad_out, false);
}

namespace {
skim_status scale_step_impl(skim_ctx *ctx, const float *W, const float *S, const float *H, int64_t n, int64_t m,
                            int64_t ld, const uint8_t *labels, float *alpha, float *adam_m, float *adam_v, int64_t t,
                            const skim_adam_opts *opts, double *loss_before, float *grad_out, bool h_ready) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!W || !S || !H || !labels || !alpha || !adam_m || !adam_v || !opts || !loss_before)
        SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_scale_step: NULL argument");
    if (t < 1 || opts->decay_every < 1) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_scale_step: t and decay_every must be >= 1");
    if ((st = check_shape(ctx, n, m, ld)) != SKIM_OK) return st;
    if ((uintptr_t)H & 15) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_scale_step: H must be 16-byte aligned");
    LossWs w;
    if ((st = carve(ctx, n, m, true, w)) != SKIM_OK) return st;
    hipLaunchKernelGGL(row_prep_kernel, dim3((unsigned)n), dim3(PREP_THREADS), 0, ctx->stream, W, S, (const float *)alpha,
                       (long long)m, (long long)ld, labels, w.cent, w.Den, w.dW, w.dWp, (const double *)nullptr, 0ll, 0,
                       rows_vec4(W, S, alpha, labels, ld));
    if ((st = launch_contraction(ctx, w, H, n, m, true, h_ready)) != SKIM_OK) return st;
    launch_loss_finish(ctx->stream, w.partial, w.ntile, (long long)n, loss_before, (double *)nullptr, 1ll);
    // rows of W, S, P start 16-byte aligned and the labels of a row 4-byte aligned (m is a multiple of 16)
    const bool vec4 = rows_vec4(W, S, alpha, labels, ld) && ((uintptr_t)w.P & 15) == 0;
    if (m <= (int64_t)GRAD_NC * PREP_THREADS)
        hipLaunchKernelGGL(grad_rows_kernel<true>, dim3(w.nstrip), dim3(PREP_THREADS), 0, ctx->stream, W, S,
                           (const float *)alpha, (long long)n, (long long)m, (long long)ld, labels, w.P, w.cent, w.Den,
                           w.gpart, vec4);
    else
        hipLaunchKernelGGL(grad_rows_kernel<false>, dim3(w.nstrip), dim3(PREP_THREADS), 0, ctx->stream, W, S,
                           (const float *)alpha, (long long)n, (long long)m, (long long)ld, labels, w.P, w.cent, w.Den,
                           w.gpart, false);
    const double lr = (double)opts->lr0 * pow((double)opts->decay, (double)((t - 1) / opts->decay_every));
    const double bc1 = 1.0 - pow((double)opts->beta1, (double)t), bc2 = 1.0 - pow((double)opts->beta2, (double)t);
    hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((m + ADAM_COLS - 1) / ADAM_COLS)), dim3(ADAM_COLS * ADAM_GROUPS), 0, ctx->stream, w.gpart, w.nstrip,
                       (long long)m, alpha, adam_m, adam_v, (float)lr, opts->beta1, opts->beta2, opts->eps, (float)bc1,
                       (float)bc2, grad_out);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}
}  // namespace

// Scaling-vector training (Alg. 2): `outer` rounds of { labels = K-means of W * alpha^-1 at the given bit
// widths; `steps` optimiser steps on alpha with the labels fixed }, then the centroids and the loss at the
// final alpha.  Composition of skim_cluster_rows, skim_scale_step and the layer-loss kernels.
extern "C" skim_status skim_train_scale(skim_ctx *ctx, const float *W, const float *S, const float *H, int64_t n,
                                        int64_t m, int64_t ld, const uint8_t *bits, int kmeans_iters, int outer,
                                        int steps, int64_t t0, const skim_adam_opts *opts, float *alpha,
                                        float *adam_m, float *adam_v, uint8_t *labels, double *centroids,
                                        double *loss_trace) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!W || !S || !H || !bits || !opts || !alpha || !adam_m || !adam_v || !labels || !centroids || !loss_trace)
        SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_train_scale: NULL argument");
    if (outer < 1 || steps < 0 || t0 < 1 || kmeans_iters < 1)
        SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_train_scale: need outer >= 1, steps >= 0, t0 >= 1, kmeans_iters >= 1");
    if (ctx->ws_bytes < skim_workspace_bytes(n, m))
        SKIM_FAIL(ctx, SKIM_ERR_WORKSPACE, "workspace missing or smaller than skim_workspace_bytes(n, m)");
    // per-row clustering outputs that the caller does not ask for live at the tail of the workspace
    // (the calls below carve from its start)
    const size_t tail_bytes = (((size_t)n * 16 * sizeof(float) + 255) & ~(size_t)255) +
                              (((size_t)n * sizeof(double) + 255) & ~(size_t)255);
    char *tail = (char *)ctx->ws + ((ctx->ws_bytes - tail_bytes) & ~(size_t)255);
    float *upper = (float *)tail;
    double *err = (double *)(tail + (((size_t)n * 16 * sizeof(float) + 255) & ~(size_t)255));
    int64_t t = t0;
    int64_t slot = 0;
    for (int round = 0; round < outer; ++round) {
        if ((st = skim_cluster_rows(ctx, W, S, alpha, n, m, ld, bits, kmeans_iters, labels, centroids, upper, err)) !=
            SKIM_OK)
            return st;
        // H is cut into its pieces once per round (the re-clustering has written over that part of the workspace)
        for (int k = 0; k < steps; ++k, ++t, ++slot) {
            if ((st = scale_step_impl(ctx, W, S, H, n, m, ld, labels, alpha, adam_m, adam_v, t, opts, loss_trace + slot,
                                      nullptr, k > 0)) != SKIM_OK)
                return st;
        }
    }
    // centroids of the fixed labels at the final alpha, and the loss there
    if ((st = check_shape(ctx, n, m, ld)) != SKIM_OK) return st;
    LossWs w;
    if ((st = carve(ctx, n, m, false, w)) != SKIM_OK) return st;
    if ((st = skim_layer_loss(ctx, W, S, alpha, H, n, m, ld, labels, loss_trace + slot, nullptr)) != SKIM_OK) return st;
    SKIM_HIP(ctx, hipMemcpyAsync(centroids, w.cent, (size_t)n * 16 * sizeof(double), hipMemcpyDeviceToDevice, ctx->stream));
    return SKIM_OK;
}
