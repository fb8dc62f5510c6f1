// Layer-wise Hessian proxy from calibration activations (Sec. 3.4: H ~ X X^T in the paper's
// column convention; here X is N x m row-major, one activation vector per row, so
// H = X^T X / N, m x m).  bf16 inputs, bf16 MFMA (v_mfma_f32_32x32x16_bf16) with float32
// accumulation over chunks of activations.  Two kernels: 128 x 128 output tiles with the chunks
// (2048 activations) added up in float64 registers, and, for layers of more than 2560 columns,
// 256 x 256 tiles (the symmetric half, mirrored at the end) with the chunks (8192 activations) added
// up in float32 in H itself.
#include "skim_common.h"
#include <type_traits>

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
// columns [cb, ce) of the task's 8 (compile-time bounds once the caller's loop is unrolled): the 8 activations of
// column 8 cg + c go to 16-byte slot `slot` of that column's LDS row
__device__ __forceinline__ void store_cols(uint16_t (*T)[HK_PAD], int cg, int slot, const Staged &s, int cb, int ce) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        if (c < cb || c >= ce) continue;
        uint32_t o[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t a = s.r[2 * d][c >> 1], b = s.r[2 * d + 1][c >> 1];
            o[d] = (c & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
        }
        *(uint4 *)&T[8 * cg + c][8 * slot] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}
__device__ __forceinline__ void store_task(XTile &T, int st, const Staged &s) { store_cols(T.t, st >> 3, st & 7, s, 0, 8); }

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

// ---- the kernel for large m: 256 x 256 output tile, one workgroup per CU, tiles on and above the diagonal only -----
// Eight wavefronts, two per SIMD, each a 128 x 64 part of the tile (4 x 2 accumulator tiles of 32 x 32), so an MFMA
// operand read from LDS feeds 2.7 MFMAs instead of two and a byte fetched from L2 feeds twice the arithmetic of the
// 128 x 128 kernel; while one wavefront of a SIMD waits for LDS, memory or the barrier the other one issues MFMAs.
// Two register sets stage the X tiles: the loads of tile kt + 2 are issued at the start of step kt and stored to
// LDS in the second half of step kt + 1, between the MFMAs of that step, so neither the memory latency nor the
// transposes stand between two steps.  The float32 accumulators are added into H itself (float32,
// read-modify-write by the one thread that owns the entry) every 8192 activations: the sums over a chunk carry at
// most 512 roundings at 1/16 or less of the total each, the 16 chunk additions of 131072 activations one rounding
// each -- a few 1e-6 of sqrt(H_jj H_ll) in the worst case.
constexpr int BT = 256;
constexpr int B_THREADS = 512;
constexpr int B_FLUSH_TILES = 128;
struct BTile {
    uint16_t t[BT][HK_PAD];
};
constexpr size_t B_LDS_BYTES = 4 * sizeof(BTile);     // two operands, double-buffered: 147456 bytes

// 16-byte loads of one task (8 activations x 8 columns) from rows k0 + 8 ab + t; CHECK: rows past N read as zero
template <bool CHECK>
__device__ __forceinline__ void load_rows(const uint16_t *__restrict__ p, long long m, long long krem, Staged &s) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (!CHECK || t < krem) v = *(const uint4 *)(p + t * m);
        s.r[t][0] = v.x; s.r[t][1] = v.y; s.r[t][2] = v.z; s.r[t][3] = v.w;
    }
}

// Needs m % 8 == 0, X 16-byte aligned (every 8-column group of a row is one aligned 16-byte load) and N >= 128.
__global__ void __launch_bounds__(B_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
xtx_big_kernel(const uint16_t *__restrict__ X, long long N, long long m, float *__restrict__ H, int nt) {
    extern __shared__ __align__(16) unsigned char smem[];
    BTile *TI = (BTile *)smem, *TJ = TI + 2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 2, wc = wave & 3;
    const int l32 = lane & 31, lhi = lane >> 5;
    // Workgroup -> tile.  H is symmetric: only the tiles (bi, bj) with bi <= bj are computed, nt (nt + 1) / 2 of them,
    // and a tile off the diagonal writes its transpose as well at the end.  Consecutive workgroup ids go to the 8
    // XCDs in turn; the ids one XCD receives are mapped to consecutive tiles of a band-by-band order (bands of 8
    // tile rows; inside a band column by column, first the columns the diagonal cuts short), so the workgroups
    // that share an L2 at any time share operand panels: 32 of them cover about 8 x 4 tiles, 12 panels for 64 uses.
    long long v = blockIdx.x;
    const long long total = (long long)nt * (nt + 1) / 2;
    {
        const long long q8 = total >> 3, r8 = total & 7, xcd = v & 7;     // XCD xcd receives q8 (+ 1 if xcd < r8) ids
        v = xcd * q8 + min(xcd, r8) + (v >> 3);
    }
    int bi = 0, bj = 0;
    for (int rb = 0; rb < nt; rb += 8) {
        const int hb = min(8, nt - rb);
        const long long tri = (long long)hb * (hb + 1) / 2, cnt = tri + (long long)hb * (nt - rb - hb);
        if (v < cnt) {
            if (v < tri) {          // column rb + t holds the t + 1 rows rb .. rb + t
                int t = 0;
                while (v >= t + 1) {
                    v -= t + 1;
                    ++t;
                }
                bj = rb + t;
                bi = rb + (int)v;
            } else {
                v -= tri;
                bj = rb + hb + (int)(v / hb);
                bi = rb + (int)(v % hb);
            }
            break;
        }
        v -= cnt;
    }
    const long long i0 = (long long)bi * BT, j0 = (long long)bj * BT;

    floatx16 acc[4][2];

    // Staging: wavefronts 0-3 move the i tile, 4-7 the j tile; a thread moves activations 8 ab .. + 7 of columns
    // 8 cg .. + 7, the 32 lanes of a half wavefront the 32 column groups of one row: a load instruction reads 512
    // contiguous bytes of each of two rows (with ab fastest it would be 128 bytes of eight rows 8 m bytes apart,
    // which the memory system serves at half the rate).  A column group past the matrix reads the tile's first
    // group instead: its products only reach entries (i >= m or j >= m) that are never stored.
    // LDS row of a column: its 64 activations as eight 16-byte slots, rotated by (column / 32) slots.  An operand
    // read (lanes = 32 consecutive columns, one rotation) then has the plain 144-byte row stride of the unrotated
    // layout, and a staging store (lanes = column groups, 8 x 144 bytes apart, which alone would fall into one set
    // of banks) spreads over the banks by its rotations: within the 32 lanes of a row the groups are dealt out
    // 0, 4, .. 28, 1, 5, .. so that any 8 consecutive lanes carry 8 different rotations.
    const int su = tid & 255;
    const bool stage_j = tid >= 256;
    const int cg = 4 * (su & 7) + ((su >> 3) & 3), ab = su >> 5;
    const int st_slot = (ab + (cg >> 2)) & 7;
    const long long sc0 = stage_j ? j0 : i0;
    const uint16_t *px = X + (long long)(8 * ab) * m + (sc0 + 8 * cg < m ? sc0 + 8 * cg : sc0);
    BTile *const ST = stage_j ? TJ : TI;
    // The activations are cut into 64-row tiles from the end: the first one is the short one, rows [0, r0) with
    // r0 = N - 64 (nreal - 1) in 1 .. 64, zero-padded to 64.  An all-zero tile goes in front when that makes the
    // count even, so the loop below runs whole pairs of steps and, from tile 2 on, loads full tiles without
    // looking at N.
    const long long nreal = (N + HK - 1) / HK;          // >= 2: the host sends N >= 128 here
    const int odd = (int)(nreal & 1);
    const long long ntile = nreal + odd;
    const long long r0 = N - (nreal - 1) * HK;
    Staged sg[2];                // two tiles on their way from global memory to LDS: tile t in set t & 1
    auto load_tile = [&](long long kt, Staged &d) {
        const long long k0 = r0 + (kt - 1 - odd) * HK;
        load_rows<false>(px + k0 * m, m, 0, d);
    };
    if (odd) {
        load_rows<true>(px, m, 0, sg[0]);                  // no rows: zeros
        load_rows<true>(px, m, r0 - 8 * ab, sg[1]);
    } else {
        load_rows<true>(px, m, r0 - 8 * ab, sg[0]);
        load_tile(1, sg[1]);
    }
    store_cols(ST[0].t, cg, st_slot, sg[0], 0, 8);
    __syncthreads();
    const double inv = 1.0 / (double)N;
    // A wavefront takes every other 32-column block of the i tile and every fourth of the j tile: rows
    // 32 (2 x + wr) + lane % 32 and 32 (4 y + wc) + lane % 32.  Operand of a lane in k-slice ks: activations
    // 16 ks + 8 (lane / 32) .. + 7, i.e. slot (2 ks + lane / 32 + block) % 8 of its row: four values per operand,
    // by (ks + x) % 4 and (ks + 2 y) % 4.
    int rslot_a[4], rslot_b[4];  // (as first activation of the slot)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        rslot_a[q] = 8 * ((2 * q + wr + lhi) & 7);
        rslot_b[q] = 8 * ((2 * q + wc + lhi) & 7);
    }

    // one step: first the loads of tile kt + 2 are issued (into the register set tile kt left when it went to LDS
    // in the step before), then the MFMAs of tile kt (LDS buffer PAR); during the second half tile kt + 1, requested
    // a step and a half ago, goes from its registers into the other buffer
    auto step = [&](auto par_c, auto fresh_c, long long kt) {
        constexpr int PAR = decltype(par_c)::value;
        constexpr bool FRESH = decltype(fresh_c)::value;     // first step of a chunk: the sums start from zero
        load_tile(min(kt + 2, ntile - 1), sg[PAR]);          // (past the end: the last tile again, unused)
#pragma unroll
        for (int ks = 0; ks < HK / 16; ++ks) {
            bf16x8 a[4], b[2];
#pragma unroll
            for (int x = 0; x < 4; ++x) a[x] = *(const bf16x8 *)&TI[PAR].t[32 * (2 * x + wr) + l32][rslot_a[(ks + x) & 3]];
#pragma unroll
            for (int y = 0; y < 2; ++y) b[y] = *(const bf16x8 *)&TJ[PAR].t[32 * (4 * y + wc) + l32][rslot_b[(ks + 2 * y) & 3]];
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y) {
                    if (FRESH && ks == 0) {
                        floatx16 zero;
#pragma unroll
                        for (int e = 0; e < 16; ++e) zero[e] = 0.f;
                        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x], b[y], zero, 0, 0, 0);
                    } else {
                        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x], b[y], acc[x][y], 0, 0, 0);
                    }
                }
            if (ks >= 2)        // (after the last tile this stores a repeat of the last tile: harmless, never read)
                store_cols(ST[PAR ^ 1].t, cg, st_slot, sg[PAR ^ 1], 4 * (ks - 2), 4 * (ks - 2) + 4);
        }
        __syncthreads();
    };
    for (long long c0 = 0; c0 < ntile; c0 += B_FLUSH_TILES) {
        const long long cend = min(c0 + (long long)B_FLUSH_TILES, ntile);
        // (c0 is even: tile kt sits in LDS buffer kt & 1)
        // (whole pairs: a second step under a condition would have the loads of the first, which only it uses,
        // sunk into that condition by the compiler, a whole step late)
        step(std::integral_constant<int, 0>{}, std::true_type{}, c0);
        step(std::integral_constant<int, 1>{}, std::false_type{}, c0 + 1);
        for (long long kt = c0 + 2; kt < cend; kt += 2) {
            step(std::integral_constant<int, 0>{}, std::false_type{}, kt);
            step(std::integral_constant<int, 1>{}, std::false_type{}, kt + 1);
        }
        // the chunk's sums go into H.  Accumulator element e of a 32 x 32 tile: row = 8*(e/4) + 4*(lane/32) + e%4,
        // column = lane%32.  Straight-line code, one accumulator tile at a time: an entry outside the matrix is
        // turned into "add nothing to this thread's first entry" instead of a branch (with a branch per entry the
        // compiler copies all accumulators out at once and spills what the MFMA loop keeps in registers).
        // (The empty asm keeps the address arithmetic of this rare block inside it.)
        const bool first = c0 == 0, last = cend == ntile;
        const long long ib = i0 + wr * 32 + 4 * lhi, jb = j0 + wc * 32 + l32;
        float *hp = H + ib * m + jb;
        long long mm = m;
        int rlim = (int)min(m - ib, 4096ll), clim = (int)min(m - jb, 4096ll);   // valid rows / columns from (ib, jb) on
        double scale = last ? inv : 1.0;
        asm volatile("" : "+v"(hp), "+s"(mm), "+v"(rlim), "+v"(clim), "+v"(scale));
        if (rlim > 0 && clim > 0) {
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int r = x * 64 + 8 * (e >> 2) + (e & 3), c = y * 128;
                        const bool valid = r < rlim && c < clim;
                        float *q = valid ? hp + r * mm + c : hp;
                        const float old = *q;
                        float av;       // read here and now, not copied out ahead with all the others
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(av) : "a"(acc[x][y][e]));
                        const float t = (first ? 0.f : old) + av;
                        *q = valid ? (float)((double)t * scale) : old;
                    }
                }
            // the transposed tile, once, from the finished entries (each thread reads back what it wrote itself)
            if (last && bi != bj) {
                float *ht = H + jb * m + ib;      // entry (jb, ib); entry (jb + c, ib + r) mirrors (ib + r, jb + c)
                for (int idx = 0; idx < 128; ++idx) {
                    const int x = idx >> 5, y = (idx >> 4) & 1, e = idx & 15;
                    const int r = x * 64 + 8 * (e >> 2) + (e & 3), c = y * 128;
                    if (r < rlim && c < clim) ht[c * mm + r] = hp[r * mm + c];
                }
            }
        }
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
    const int vec = (m % 8 == 0) && (((uintptr_t)X_bf16 & 15) == 0);     // rows of X start 16-byte aligned
    // 256 x 256 tiles from 11 tiles a side (m > 2560): a single round of them on a partly filled chip already beats
    // the 128 x 128 kernel there
    const long long ntb = (m + BT - 1) / BT;
    if (vec && N >= 2 * HK && ntb >= 11) {
        if (ctx->xtx_lds_enabled < 2) {
            SKIM_HIP(ctx, hipFuncSetAttribute((const void *)xtx_big_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)B_LDS_BYTES));
            SKIM_HIP(ctx, hipFuncSetAttribute((const void *)xtx_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)H_LDS_BYTES));
            ctx->xtx_lds_enabled = 2;
        }
        hipLaunchKernelGGL(xtx_big_kernel, dim3((unsigned)(ntb * (ntb + 1) / 2)), dim3(B_THREADS), B_LDS_BYTES, ctx->stream, X_bf16,
                           (long long)N, (long long)m, H, (int)ntb);
        SKIM_HIP(ctx, hipGetLastError());
        return SKIM_OK;
    }
    const unsigned nt = (unsigned)((m + HT - 1) / HT);
    hipLaunchKernelGGL(xtx_kernel, dim3(nt, nt), dim3(H_THREADS), H_LDS_BYTES, ctx->stream, X_bf16, (long long)N,
                       (long long)m, H, vec);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}
