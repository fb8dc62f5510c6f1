// Per-row sensitivity-weighted 1-D K-means (Alg. 3, pre-recording loop and 12-15; the
// re-clustering of W * alpha^-1 in Alg. 2) for gfx950.
//
// Three kernels per call.
//  sort_kernel       one workgroup per row at a time: the row's (w~, s~) pairs become 64-bit keys
//                    whose bit pattern, read as a float64, orders like (w~, s~); they are sorted
//                    once in LDS (counting sort by value bin + two register passes; a bitonic
//                    network for the rows that overflow a bin; compare-exchange = v_min_f64 +
//                    v_max_f64) and written to scratch together with float64 sums of s~, s~ w~ and
//                    s~ w~^2 per aligned 16-key chunk and the weight of every chunk's first key.
//  lloyd_iter_kernel one lane per cluster, two rows per wavefront, all four bit widths at once.
//                    In sorted order every cluster of a 1-D K-means is a contiguous rank range,
//                    so one Lloyd iteration is: per pair of neighbouring centroids a search for
//                    the rank where the nearer centroid changes (chunk by a search in LDS, rank
//                    inside the chunk from its keys), then centroid = (sum of s~ w~) / (sum of
//                    s~) over the range, assembled from the keys of the boundary chunks, a few
//                    chunk sums and a difference of double-double running sums.  In table mode it
//                    also writes centroids, bounds and errors.
//  finish_kernel     one workgroup per row: errors the iteration kernel flagged (direct evaluation
//                    over the sorted keys); for skim_cluster_rows centroids, thresholds, labels.
//
// Arithmetic on every decision path is float64 and uses the same predicates as the
// definition: |w - c_lo| versus |w - c_hi| with the lower cluster index winning equal
// distances; centroids with no weight mass keep their value.
#include "skim_common.h"

#include <math.h>

#include <type_traits>

typedef unsigned long long u64;

namespace {

constexpr int EPT = 16;           // sorted elements owned by one thread
constexpr int MIN_THREADS = 64;
constexpr int SORT_MAX_KEYS = 16384;  // keys one workgroup sorts in LDS (128 KB)
constexpr u64 NEUTRAL_KEY = 0ull;                    // encodes (w = +0, s = +0)
constexpr u64 PAD_KEY = 0x7FF0000000000000ull;       // +infinity: above every key of finite w

struct BitState;

struct ClusterParams {
    const float *W, *S, *alpha;
    long long ld;
    int m, P, logP;
    int iters;
    int bmin, bmax;       // table mode
    const uint8_t *bits;  // rows mode when non-null
    double *E;            // table: n x nb ; rows: n
    double *cent;         // table: n x stride ; rows: n x 16
    float *upper;         // same layout as cent, may be null
    uint8_t *labels;      // rows mode only, may be null
    int stride;           // entries per row in cent/upper
    // scratch written by sort_kernel, read by the Lloyd kernels (per row: m keys, n1 chunk sums and first weights)
    u64 *keys;
    double2 *L1;          // (sum of s, sum of s*w) of every 16-key chunk (n1 per row)
    double2 *Q;           // the same sums over every group of 4 chunks (nq = n1 / 4 per row)
    int nq;
    double *R1, *RQ;      // sum of s*w*w of every chunk (n1 per row) and of every group of 4 chunks (nq per row)
    float *w16;           // weight of the first key of every 16-key chunk (n1 per row)
    BitState *bstate;  // final state of the Lloyd lanes: 4 per row (bit widths 1..4)
    int n1;
    // rows longer than one LDS sort are sorted in nseg segments of seglen columns (keys_seg),
    // merged into keys, and their sums are taken by a separate kernel
    int nseg, seglen;
    u64 *keys_seg;
    int *segmass;         // per segment of a long row: nonzero when it holds sensitivity mass
    long long nwork;      // rows x segments: the units of work sort_kernel's workgroups share out
    int *work_counters;   // [0] units handed out beyond every workgroup's first two, [1] workgroups done (both zero at launch)
    int *vflag;           // validation result (one word of scratch)
    // bucket path of sort_kernel: value bins per thread (0: always the bitonic network) and the byte
    // offsets of its tables inside the dynamic LDS
    int bk_bpt;
    int bk_pad, bk_lgbpt;   // spare words after every thread's block of counters (0 or 4); log2(bk_bpt) when padded
    uint32_t bk_hist_off, bk_coarse_off, bk_misc_off;
};

struct BitState {  // what the Lloyd lanes of one bit width leave for the epilogue
    double cent[16];  // by sorted position
    int idx[16];      // cluster index at that position
    int B[17];        // first rank of each position's range, B[K] = m
    int active;
    double err;       // row error from the clusters' second moments
    int exact;        // nonzero: err lost too many digits to cancellation, evaluate it key by key
    int pad_;
};

// LDS slot of key index i: one spare slot after every 16 keys.  The skew makes the access patterns
// of all passes (almost) free of bank conflicts, and it is additive: the 16 keys of a thread that
// differ in index bits [wb, wb+4) sit at a fixed stride, so their addresses are one per-thread base
// plus compile-time offsets that go into the instructions' offset fields.
__device__ __forceinline__ uint32_t swz(uint32_t i) { return i + (i >> 4); }

// Key of a (w, s) pair, s >= 0, both finite.  High word = the bits of w (-0 folded into +0), low
// word = the bits of s, complemented when w is negative.  Read as a float64 the key is finite
// (its exponent field is all ones only for w = inf/nan) and orders like (w, s): positive keys
// grow with (high, low); negative keys fall with their magnitude, i.e. with |w| and, for equal
// w, with the complemented s.  Two keys are equal only when w and s are.
__device__ __forceinline__ u64 make_key(float w, float s) {
    w = __fadd_rn(w, 0.0f);   // -0 + 0 = +0 under round-to-nearest; every other value is unchanged
    s = __fadd_rn(s, 0.0f);
    const uint32_t hi = __float_as_uint(w);
    uint32_t lo = __float_as_uint(s);
    if (hi >> 31) lo = ~lo;
    return ((u64)hi << 32) | (u64)lo;
}
__device__ __forceinline__ float elem_w(u64 e) { return __uint_as_float((uint32_t)(e >> 32)); }
__device__ __forceinline__ float elem_s(u64 e) {
    const uint32_t lo = (uint32_t)e;
    return __uint_as_float((e >> 63) ? ~lo : lo);
}
// The sorted keys in global memory (ClusterParams::keys) carry s as it is: the complement only serves the order
// inside the sort, and the kernels that read the sorted rows would undo it for every key they touch.
__device__ __forceinline__ u64 plain_key(u64 e) { return (e >> 63) ? (e ^ 0xFFFFFFFFull) : e; }
__device__ __forceinline__ float plain_s(u64 e) { return __uint_as_float((uint32_t)e); }
// same key with s replaced by 1 (unit weights)
__device__ __forceinline__ u64 unit_weight_key(u64 e) {
    const uint32_t one = 0x3F800000u;
    return (e & 0xFFFFFFFF00000000ull) | (u64)((e >> 63) ? ~one : one);
}

// Column scaling ahead of the clustering (Sec. 4.3): w~ = w / alpha and
// s~ = (s * alpha) * alpha, each a single-precision IEEE operation.
__device__ __forceinline__ void scaled_pair(float w, float s, const float *alpha, int j, float &wt, float &st) {
    if (alpha) {
        const float a = alpha[j];
        wt = __fdiv_rn(w, a);
        st = __fmul_rn(__fmul_rn(s, a), a);
    } else {
        wt = w;
        st = s;
    }
}

// Compare-exchange, smaller key to a: two full-rate VALU instructions on the float64 view of
// the keys (min/max return one of their finite operands bit for bit).
__device__ __forceinline__ void ce(double &a, double &b) {
    double lo, hi;
    asm("v_min_f64 %0, %1, %2" : "=v"(lo) : "v"(a), "v"(b));
    asm("v_max_f64 %0, %1, %2" : "=v"(hi) : "v"(a), "v"(b));
    a = lo;
    b = hi;
}

// Bitonic sorting network in its direction-free form: the merge of size 2^klog starts with a
// "flip" stage that pairs index i with i ^ (2^klog - 1), followed by the stages i <-> i ^ 2^b for
// b = klog-2 .. 0; every comparator sends the smaller key to the lower index.  Padding keys
// (+inf at the top indices) therefore never move.
//
// One pass over LDS: the thread holds the 16 keys whose indices differ in bits [WB, WB+4) and
// runs up to 4 consecutive stages in registers.  In a pass that opens a merge (FLIP >= 0 is the
// window bit of the flip stage) the registers with that bit set are taken from the thread whose
// low WB index bits are complemented, so that both keys of every flip pair sit in one thread.
// Stages run on window bits HI .. LO after the flip stage.
typedef __attribute__((address_space(3))) volatile double lds_vdouble;
typedef __attribute__((address_space(3))) char lds_char;

template <int WB, int FLIP, int HI, int LO>
__device__ __forceinline__ void sort_pass(double *lds, uint32_t t, int m) {
    static_assert(WB == 0 || WB >= 4, "window below bit 4 must start at bit 0");
    constexpr uint32_t lowmask = (1u << WB) - 1u;
    constexpr uint32_t STRIDE = ((1u << WB) + (WB >= 4 ? (1u << (WB - 4)) : 0u)) * 8u;   // bytes between registers
    constexpr int FB = FLIP >= 0 ? FLIP : 0;
    const uint32_t base = ((t >> WB) << (WB + 4)) | (t & lowmask);
    if ((int)(base & ~lowmask) >= m) return;   // all 16 keys are padding
    lds_char *const pa = (lds_char *)lds + swz(base) * 8u;
    lds_char *const pf = (lds_char *)lds + swz(base ^ lowmask) * 8u;
    double v[EPT];
#pragma unroll
    for (int r = 0; r < EPT; ++r) {
        const bool flipped = (FLIP >= 0) && (r & (1 << FB));
        // (volatile keeps 16 single 8-byte accesses: the paired ds_read2/ds_write2 forms the
        // compiler would merge them into move fewer bytes per clock on this LDS)
        v[r] = *(lds_vdouble *)((flipped ? pf : pa) + r * STRIDE);
    }
    if (FLIP >= 0) {
#pragma unroll
        for (int r = 0; r < EPT; ++r)
            if (!(r & (1 << FB))) ce(v[r], v[r ^ ((2 << FB) - 1)]);
    }
#pragma unroll
    for (int rb = HI; rb >= LO; --rb) {
#pragma unroll
        for (int r = 0; r < EPT; ++r)
            if (!(r & (1 << rb))) ce(v[r], v[r | (1 << rb)]);
    }
#pragma unroll
    for (int r = 0; r < EPT; ++r) {
        const bool flipped = (FLIP >= 0) && (r & (1 << FB));
        *(lds_vdouble *)((flipped ? pf : pa) + r * STRIDE) = v[r];
    }
}

// The merges of size 2, 4, 8, 16 in one pass (index bits 0..3 are in-thread).
__device__ __forceinline__ void sort_first_pass(double *lds, uint32_t t, int m) {
    const uint32_t base = t << 4;
    if ((int)base >= m) return;
    lds_vdouble *const pa = (lds_vdouble *)lds + swz(base);
    double v[EPT];
#pragma unroll
    for (int r = 0; r < EPT; ++r) v[r] = pa[r];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
#pragma unroll
        for (int r = 0; r < EPT; ++r)
            if (!(r & (1 << tb))) ce(v[r], v[r ^ ((2 << tb) - 1)]);
#pragma unroll
        for (int rb = tb - 1; rb >= 0; --rb) {
#pragma unroll
            for (int r = 0; r < EPT; ++r)
                if (!(r & (1 << rb))) ce(v[r], v[r | (1 << rb)]);
        }
    }
#pragma unroll
    for (int r = 0; r < EPT; ++r) pa[r] = v[r];
}

// The last stages of a merge, index bits 9..0, inside the 1024 keys a wavefront owns (windows
// [6,10) for bits 9..8, [4,8) for bits 7..4, [0,4) for bits 3..0): no workgroup barrier is needed
// between these passes, because a wavefront's LDS accesses execute in order.
__device__ __forceinline__ void wave_tail(double *lds, uint32_t tid, int m) {
    sort_pass<6, -1, 3, 2>(lds, tid, m);
    sort_pass<4, -1, 3, 0>(lds, tid, m);
    sort_pass<0, -1, 3, 0>(lds, tid, m);
}

// Merges of 2^KLOG > 1024 keys.  KLOG = 11, 12 (11 and 12 stages) take three passes: the window
// [KLOG-4, KLOG) between two workgroup barriers (flip stage on index bit KLOG-1 and the three bits below
// it), then the windows [4,8) and [0,4) inside the wavefront's own 1024 keys.  KLOG = 13, 14 need four:
// the top window [LOGP-4, LOGP) between barriers (flip stage, then the bits down to 10), then wave_tail.
template <int LOGP, int KLOG>
__device__ __forceinline__ void cross_merges(double *lds, uint32_t tid, int m) {
    if constexpr (KLOG <= LOGP) {
        if constexpr (KLOG <= 12) {
            __syncthreads();
            sort_pass<KLOG - 4, 3, 2, 0>(lds, tid, m);          // index bits KLOG-1 .. KLOG-4
            __syncthreads();
            sort_pass<4, -1, KLOG - 9, 0>(lds, tid, m);         // index bits KLOG-5 .. 4
            sort_pass<0, -1, 3, 0>(lds, tid, m);
        } else {
            constexpr int WBX = LOGP - 4;
            __syncthreads();
            sort_pass<WBX, KLOG - 1 - WBX, KLOG - 2 - WBX, 10 - WBX>(lds, tid, m);
            __syncthreads();
            wave_tail(lds, tid, m);
        }
        cross_merges<LOGP, KLOG + 1>(lds, tid, m);
    }
}

// Sort of P = 2^LOGP >= 1024 keys in LDS (the last P - m of them padding) by P/16 threads.
// Merges up to 1024 keys run inside one wavefront (its 64 threads own an aligned block of 1024
// keys); every pass has its window, its stages and hence its LDS offsets fixed at compile time.
template <int LOGP>
__device__ __forceinline__ void sort_row(double *lds, uint32_t tid, int m) {
    sort_first_pass(lds, tid, m);
    sort_pass<4, 0, -1, 0>(lds, tid, m);    // merges of 32 keys
    sort_pass<0, -1, 3, 0>(lds, tid, m);
    sort_pass<4, 1, 0, 0>(lds, tid, m);     // 64
    sort_pass<0, -1, 3, 0>(lds, tid, m);
    sort_pass<4, 2, 1, 0>(lds, tid, m);     // 128
    sort_pass<0, -1, 3, 0>(lds, tid, m);
    sort_pass<4, 3, 2, 0>(lds, tid, m);     // 256
    sort_pass<0, -1, 3, 0>(lds, tid, m);
    sort_pass<6, 2, 1, 2>(lds, tid, m);     // 512: bit 8 in the window [6,10)
    sort_pass<4, -1, 3, 0>(lds, tid, m);
    sort_pass<0, -1, 3, 0>(lds, tid, m);
    sort_pass<6, 3, 2, 2>(lds, tid, m);     // 1024: bits 9..8
    sort_pass<4, -1, 3, 0>(lds, tid, m);
    sort_pass<0, -1, 3, 0>(lds, tid, m);
    cross_merges<LOGP, 11>(lds, tid, m);
    __syncthreads();
}

__device__ __forceinline__ double shfl_d(double x, int src) { return __shfl(x, src, 64); }

// Cross-lane moves that stay inside the VALU (DPP): lane i reads lane i^1 / lane i^2.
template <int CTRL>
__device__ __forceinline__ int dpp_move_i(int x) {
    return __builtin_amdgcn_update_dpp(x, x, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ double dpp_move_d(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = dpp_move_i<CTRL>(lo);
    hi = dpp_move_i<CTRL>(hi);
    return __hiloint2double(hi, lo);
}
// Neighbouring lanes of the whole wavefront inside the VALU: lane i reads lane i-1 / lane i+1
// (lane 0 / lane 63 keep their own value).
__device__ __forceinline__ int lane_below(int x) { return __builtin_amdgcn_update_dpp(x, x, 0x138, 0xF, 0xF, false); }
__device__ __forceinline__ int lane_above(int x) { return __builtin_amdgcn_update_dpp(x, x, 0x130, 0xF, 0xF, false); }
__device__ __forceinline__ double lane_below(double x) {
    return __hiloint2double(lane_below(__double2hiint(x)), lane_below(__double2loint(x)));
}
__device__ __forceinline__ double lane_above(double x) {
    return __hiloint2double(lane_above(__double2hiint(x)), lane_above(__double2loint(x)));
}
// Sum over the four lanes of a quad; every lane of the quad gets the same bits.
__device__ __forceinline__ double quad_sum(double x) {
    x += dpp_move_d<0xB1>(x);  // quad_perm [1,0,3,2]
    x += dpp_move_d<0x4E>(x);  // quad_perm [2,3,0,1]
    return x;
}
__device__ __forceinline__ int quad_sum(int x) {
    x += dpp_move_i<0xB1>(x);
    x += dpp_move_i<0x4E>(x);
    return x;
}

// ---------------------------------------------------------------------------------------------
// Bucket path of the sort.  A full sorting network pays for the worst case; the rows here are m
// draws from a smooth density, so a monotone map from the weight to one of about 1.5 m value bins
// leaves a handful of keys per bin, and a counting sort by bin puts every key within a few slots
// of its final rank in one scatter.  What remains is order inside the bins:
//   * every thread sorts the 16 slots [16t, 16t+16) in registers (Batcher's odd-even merge sort,
//     63 compare-exchanges), which orders every bin that lies inside one such window;
//   * a bin that straddles a multiple of 16 has at most 8 keys on either side when no bin holds
//     more than 9 keys, so one 8+8 merge of the upper half of window t with the lower half of
//     window t+1 (25 compare-exchanges) finishes the row.
// The bin map has two levels so that it adapts to the row: a coarse histogram over COARSE_N equal
// intervals of [min, max], then every coarse interval is cut into a number of equal bins
// proportional to its count (a piecewise linear estimate of the distribution function).  Any
// monotone map gives a correct sort; the map only decides how full the bins get.
//   * A row in which some bin holds 10 to 17 keys (a few rows in a thousand: the map is an estimate) gets a third
//     pass, an 8+8 merge of the two halves of every window: a bin of at most 17 keys touches at most three
//     aligned blocks of 8 slots, and block merges over the pairs (2i, 2i+1), (2i+1, 2i+2), (2i, 2i+1) carry every
//     key across the two block borders it may have to cross, in either direction.
// A row in which some bin holds more than 17 keys (heavy duplicates, wild outliers, a constant row) takes the
// bitonic network instead: same result, key for key.
// ---------------------------------------------------------------------------------------------
// (a bin of 9 keys that straddles a multiple of 16 still has at most 8 on either side, one of 10 may have 9;
// likewise 17 for three passes)
constexpr int BIN_MAX_KEYS = 9;      // no bin above this: two passes
constexpr int BIN_MAX_KEYS3 = 17;    // no bin above this: three passes

// position of a weight on the coarse axis; single-precision operations that the compiler may not fuse,
// so that the two places that evaluate it agree bit for bit
__device__ __forceinline__ float coarse_pos(float w, float lo, float scale) { return __fmul_rn(__fsub_rn(w, lo), scale); }

#define SKIM_X(a, b) ce(v[a], v[b]);
// Batcher's odd-even merge sort of 16 keys, in layers of independent comparators
__device__ __forceinline__ void sort16(double (&v)[16]) {
    SKIM_X(0,1) SKIM_X(2,3) SKIM_X(4,5) SKIM_X(6,7) SKIM_X(8,9) SKIM_X(10,11) SKIM_X(12,13) SKIM_X(14,15)
    SKIM_X(0,2) SKIM_X(1,3) SKIM_X(4,6) SKIM_X(5,7) SKIM_X(8,10) SKIM_X(9,11) SKIM_X(12,14) SKIM_X(13,15)
    SKIM_X(1,2) SKIM_X(5,6) SKIM_X(0,4) SKIM_X(3,7) SKIM_X(9,10) SKIM_X(13,14) SKIM_X(8,12) SKIM_X(11,15)
    SKIM_X(2,6) SKIM_X(1,5) SKIM_X(10,14) SKIM_X(9,13) SKIM_X(0,8) SKIM_X(7,15)
    SKIM_X(2,4) SKIM_X(3,5) SKIM_X(10,12) SKIM_X(11,13)
    SKIM_X(1,2) SKIM_X(3,4) SKIM_X(5,6) SKIM_X(9,10) SKIM_X(11,12) SKIM_X(13,14)
    SKIM_X(4,12) SKIM_X(2,10) SKIM_X(6,14) SKIM_X(1,9) SKIM_X(5,13) SKIM_X(3,11)
    SKIM_X(4,8) SKIM_X(6,10) SKIM_X(5,9) SKIM_X(7,11)
    SKIM_X(2,4) SKIM_X(6,8) SKIM_X(10,12) SKIM_X(3,5) SKIM_X(7,9) SKIM_X(11,13)
    SKIM_X(1,2) SKIM_X(3,4) SKIM_X(5,6) SKIM_X(7,8) SKIM_X(9,10) SKIM_X(11,12) SKIM_X(13,14)
}
// odd-even merge of v[0..8) and v[8..16), each ascending
__device__ __forceinline__ void merge8x8(double (&v)[16]) {
    SKIM_X(0,8) SKIM_X(4,12) SKIM_X(2,10) SKIM_X(6,14) SKIM_X(1,9) SKIM_X(5,13) SKIM_X(3,11) SKIM_X(7,15)
    SKIM_X(4,8) SKIM_X(6,10) SKIM_X(5,9) SKIM_X(7,11)
    SKIM_X(2,4) SKIM_X(6,8) SKIM_X(10,12) SKIM_X(3,5) SKIM_X(7,9) SKIM_X(11,13)
    SKIM_X(1,2) SKIM_X(3,4) SKIM_X(5,6) SKIM_X(7,8) SKIM_X(9,10) SKIM_X(11,12) SKIM_X(13,14)
}
#undef SKIM_X

// Inclusive prefix sum over the 64 lanes of a wavefront inside the VALU: shifts by 1, 2, 4, 8 within each
// row of 16 lanes (a lane without a source adds 0), then the last lane of row 0 / 2 into rows 1 / 3 and lane
// 31 into the upper half.
__device__ __forceinline__ uint32_t wave_scan_incl(uint32_t x) {
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xF, 0xF, false);   // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xF, 0xF, false);   // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xF, 0xF, false);   // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xF, 0xF, false);   // row_shr:8
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1, 3
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2, 3
    return x;
}
// Which of a thread's key slots hold a key of the unit, and which column a slot is.
//   VEC == false: slot k is column tid + k * nth, so all slots below kfull = m / nth hold a key, slot kfull does in
//                 the threads below m % nth, and none above.
//   VEC == true:  slots 4g .. 4g+3 are the four columns from 4 (tid + g * nth) on (one 16-byte load each of W and
//                 S); m is a multiple of 4 then and the same rule holds for g with m / 4.
// nth is a power of two, so the first test is on uniform values only.
template <bool VEC>
struct Slots {
    int kfull, tid, nth;
    bool part;
    __device__ __forceinline__ Slots(int m, int nth_, int tid_) : tid(tid_), nth(nth_) {
        const int sh = 31 - __builtin_clz((unsigned)nth_);
        const int units = VEC ? (m >> 2) : m;
        kfull = units >> sh;
        part = tid_ < (units & (nth_ - 1));
    }
    __device__ __forceinline__ bool has(int k) const {
        const int g = VEC ? (k >> 2) : k;
        return g < kfull || (g == kfull && part);
    }
    __device__ __forceinline__ int col(int k) const { return VEC ? 4 * (tid + (k >> 2) * nth) + (k & 3) : tid + k * nth; }
};

// LDS tables of the bucket path (byte offsets from ClusterParams::bk_*_off):
//   hist     two 16-bit counters per word, one per value bin; later the first rank of every bin.  A thread
//            scans the bk_bpt bins [tid * bk_bpt, (tid + 1) * bk_bpt) with 16-byte accesses; its block of words is
//            followed by bk_pad spare words so that the blocks of 8 neighbouring threads start in different banks
//   coarse   COARSE_N intervals x 4 counters (a lane adds to copy lane & 3: fewer same-address collisions),
//            then per interval (first bin, number of bins) as two floats
//   misc     per wavefront: least weight, largest weight, mass flag, OR of the weights' bits, scan total with its
//            flags, sum and count of the exponents of s (16 entries each); the fill table of BinMap (65 words)
constexpr int COARSE_N = 256;
constexpr uint32_t BK_COARSE_BYTES = COARSE_N * 4 * 4 + COARSE_N * 8;
constexpr uint32_t BK_MISC_BYTES = 1024;
constexpr uint32_t BK_WMIN = 0, BK_WMAX = 64, BK_WMASS = 128, BK_WOR = 192, BK_WTOT = 256, BK_SMIN = 320, BK_SMAX = 384, BK_STAB = 512;
constexpr int STAB_N = 64;        // pieces of the fill table: a quarter octave of s each, 8 octaves to either side of sbm

// The bin map a workgroup carries from one unit to the next: the axis of the coarse intervals and whether the
// table in LDS (bins per interval) is valid and the fine counters are zero.  The first unit of a workgroup
// builds the map from its own keys; every later unit is binned with the map the unit before it
// left behind, whose table was re-derived from that unit's exact counts -- rows of one matrix resemble each
// other, and any monotone map sorts correctly.  A unit that overflows a bin (it then sorts by the network)
// drops the map, and the next unit builds its own.
struct BinMap {
    bool have;
    float lo, scale;
    // Rows whose weights all have their low bits clear (values converted from a 16-bit format) hold every value
    // many times over, and equal weights would share one bin.  The bin is then taken from the weight with those
    // bits filled in from s: a value between this weight and the next one the format has, rising with s -- so the
    // map stays monotone in the key and equal weights spread over the bins up to the next value.  The fill is a
    // piecewise linear function of the bit pattern of s (about its logarithm): STAB_N pieces of a quarter octave
    // around sbm, the pattern in the middle of the row's mean octave; the table in LDS holds, per piece, the
    // share of the row's s below it, scaled to the 2^kz fill values (so equal weights spread evenly whatever the
    // distribution of s); s beyond the table takes the nearest end.  Integer arithmetic on a nondecreasing table:
    // monotone by construction.  lowmask = 2^kz - 1 (the clear bits, 8 to 16 of them); 0: off.
    uint32_t lowmask, sbm;
};

// The weight a key is binned by (see BinMap).  A negative weight gets the complement of the fill: its value
// must rise with s too, i.e. its magnitude fall.
// piece of the fill table a pattern of s falls into, and its position inside the piece in 2^-16ths
__device__ __forceinline__ void fill_piece(uint32_t sb, uint32_t sbm, int &idx, uint32_t &f16) {
    const int z = (int)(sb - sbm);                            // (patterns of s >= 0 are below 2^31: no wrap)
    const int q = (z >> 21) + STAB_N / 2;                     // quarter octaves; floor for negative z
    idx = min(max(q, 0), STAB_N - 1);
    f16 = q < 0 ? 0u : (q >= STAB_N ? 0xFFFFu : ((uint32_t)z & 0x1FFFFFu) >> 5);
}

template <bool SPREAD>
__device__ __forceinline__ float bin_weight(u64 key, const BinMap &map, const uint32_t *stab) {
    const uint32_t hi = (uint32_t)(key >> 32);
    if (!SPREAD) return __uint_as_float(hi);
    const uint32_t lo = (uint32_t)key;
    const bool neg = (hi >> 31) != 0u;
    const uint32_t sb = neg ? ~lo : lo;                       // the bits of s
    int idx;
    uint32_t f16;
    fill_piece(sb, map.sbm, idx, f16);
    const uint32_t t0 = stab[idx], t1 = stab[idx + 1];
    const uint32_t u = min(t0 + (((t1 - t0) * f16) >> 16), map.lowmask);
    return __uint_as_float(hi | (neg ? map.lowmask - u : u));
}

// Bins per coarse interval from the counts c[0..3] of this lane's 4 intervals (lane l: intervals 4l .. 4l+3;
// all 64 lanes call): counts smoothed (1 2 1) so that a sparse interval still gets bins from its neighbours'
// counts, one bin on top of every interval's share, running sum over the intervals = first bin.
// ratio4 = (bins to hand out) / (4 x sum of the counts).
__device__ __forceinline__ void write_bin_table(float2 *table, int lane, const float (&c)[4], float ratio4) {
    float below = __int_as_float(lane_below(__float_as_int(c[3])));
    float above = __int_as_float(lane_above(__float_as_int(c[0])));
    if (lane == 0) below = c[0];
    if (lane == 63) above = c[3];
    uint32_t ns[4];
    ns[0] = (uint32_t)((below + 2.0f * c[0] + c[1]) * ratio4) + 1u;
    ns[1] = (uint32_t)((c[0] + 2.0f * c[1] + c[2]) * ratio4) + 1u;
    ns[2] = (uint32_t)((c[1] + 2.0f * c[2] + c[3]) * ratio4) + 1u;
    ns[3] = (uint32_t)((c[2] + 2.0f * c[3] + above) * ratio4) + 1u;
    const uint32_t tot = ns[0] + ns[1] + ns[2] + ns[3];
    uint32_t base = wave_scan_incl(tot) - tot;
    float4 e0, e1;          // integers below 2^16: exact as floats
    e0.x = (float)base;
    e0.y = (float)ns[0];
    base += ns[0];
    e0.z = (float)base;
    e0.w = (float)ns[1];
    base += ns[1];
    e1.x = (float)base;
    e1.y = (float)ns[2];
    base += ns[2];
    e1.z = (float)base;
    e1.w = (float)ns[3];
    ((float4 *)table)[2 * lane] = e0;
    ((float4 *)table)[2 * lane + 1] = e1;
}

// Sorts the m keys held in registers (key[k], k < NS, the slots of Slots<VEC>) into LDS, rank r at slot
// swz(r), by the bucket path.  map: see BinMap; when map.have is false, map.lo / map.scale must hold the axis of
// this unit (least weight, COARSE_N / range) and the coarse counters must be zero (with a barrier between
// clearing them and this call).  Returns false, with nothing of value in LDS and map.have false, when some bin
// took more than BIN_MAX_KEYS3 keys; all threads of the workgroup return the same.  Contains workgroup
// barriers: every thread must call it.  wave_mass: whether a key of this wavefront carries sensitivity mass;
// anymass (out): whether any key of the unit does; a unit without mass is scattered with unit weights (single
// segment rows only).  prefetch(g), g = 1, 2, 3: issues part g of the loads of the next unit.  The parts are
// spread over the phases: all compute units run these phases nearly in step, and loads issued together by all
// of them queue up behind the memory's peak rate.
template <int NS, bool VEC, typename Prefetch>
__device__ __forceinline__ bool bucket_sort(unsigned char *smem, const ClusterParams &prm, const u64 (&key)[NS],
                                            int tid, int nth, int m, BinMap &map, bool wave_mass, int &anymass,
                                            Prefetch prefetch) {
    const int lane = tid & 63, wave = tid >> 6, nw = nth >> 6;
    const Slots<VEC> sm(m, nth, tid);
    uint32_t *hist = (uint32_t *)(smem + prm.bk_hist_off);
    uint32_t *coarse = (uint32_t *)(smem + prm.bk_coarse_off);
    float2 *table = (float2 *)(coarse + COARSE_N * 4);
    uint32_t *wtot = (uint32_t *)(smem + prm.bk_misc_off + BK_WTOT);
    const uint32_t *stab = (const uint32_t *)(smem + prm.bk_misc_off + BK_STAB);
    const int bpt = prm.bk_bpt;
    const int nbins = bpt * nth;
    const int hstride = (bpt >> 1) + prm.bk_pad;    // words from one thread's block of counters to the next
    const float lo = map.lo, scale = map.scale;
    // half-word (16-bit counter, later first rank) of a bin inside hist
    auto bin_halfword = [&](uint32_t fb) -> uint32_t {
        // (word = fb / 2 + 4 spare words per block of bk_bpt bins, half-word = 2 * word + fb % 2)
        return fb + (prm.bk_pad ? (fb >> prm.bk_lgbpt) << 3 : 0u);
    };
    if (__builtin_expect(!map.have, 0)) {
        // ---- coarse histogram of the unit's keys (a sample of every fourth key was tried: its table overflowed a
        // bin several times as often, and a unit that takes the network leaves the next without a map again)
#pragma unroll
        for (int k = 0; k < NS; ++k) {
            if (sm.has(k)) {
                const float wb = map.lowmask ? bin_weight<true>(key[k], map, stab) : bin_weight<false>(key[k], map, stab);
                const int cb = min(max((int)coarse_pos(wb, lo, scale), 0), COARSE_N - 1);
                atomicAdd(&coarse[cb * 4 + (lane & 3)], 1u);
            }
        }
        // clear this thread's share of the fine counters meanwhile
        {
            uint4 *hz = (uint4 *)(hist + tid * hstride);
            for (int q = 0; q < (bpt >> 3); ++q) hz[q] = make_uint4(0u, 0u, 0u, 0u);
        }
        __syncthreads();
        // ---- the table.  Every wavefront works the whole table out for itself (4 intervals per lane) and writes
        // it: all write the same words, and a wavefront's own LDS accesses execute in order, so no barrier is
        // needed before the table is used.
        const uint4 *cc4 = (const uint4 *)coarse;
        float c[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint4 t = cc4[4 * lane + q];
            c[q] = (float)(t.x + t.y + t.z + t.w);
        }
        write_bin_table(table, lane, c, (float)(nbins - COARSE_N - 16) / (4.0f * (float)m));
    }
    // ---- fine bin of every key; the counter's old value is the key's slot inside its bin
    uint32_t fbs[NS];
    uint32_t smax = 0;          // largest slot any of this thread's keys got
    const bool padded = prm.bk_pad != 0;
    auto count_keys = [&](auto spread) {
        constexpr bool SPREAD = decltype(spread)::value;
        if (sm.has(NS - 1)) {
            // every slot of this thread holds a key (all threads of a full wavefront): the same steps as below,
            // but half the slots at a time and step by step, so that the LDS reads of a batch are in flight
            // together and then its atomics (key by key, every LDS access waits for the one before it)
            constexpr int HB = NS / 2;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float fr[HB];
                uint32_t cb[HB];
#pragma unroll
                for (int i = 0; i < HB; ++i) {
                    const int k = h * HB + i;
                    const float x = fminf(fmaxf(coarse_pos(bin_weight<SPREAD>(key[k], map, stab), lo, scale), 0.0f), (float)COARSE_N - 0.0001f);
                    if (SPREAD && ((uint32_t)(key[k] >> 32) & map.lowmask)) smax = (uint32_t)BIN_MAX_KEYS3;
                    cb[i] = (uint32_t)(int)x;
                    fr[i] = __builtin_amdgcn_fractf(x);
                }
                float2 tb[HB];
#pragma unroll
                for (int i = 0; i < HB; ++i) tb[i] = table[cb[i]];
                uint32_t hw[HB], old[HB];
#pragma unroll
                for (int i = 0; i < HB; ++i) {
                    const uint32_t fb = min((uint32_t)fmaf(fr[i], tb[i].y, tb[i].x), (uint32_t)(nbins - 1));
                    hw[i] = padded ? bin_halfword(fb) : fb;
                    old[i] = atomicAdd(&hist[hw[i] >> 1], 1u << ((hw[i] & 1u) << 4));
                }
#pragma unroll
                for (int i = 0; i < HB; ++i) {
                    const uint32_t slot = (old[i] >> ((hw[i] & 1u) << 4)) & 0xFFFFu;
                    smax = max(smax, slot);
                    fbs[h * HB + i] = hw[i] | (slot << 16);
                }
            }
            return;
        }
#pragma unroll
        for (int k = 0; k < NS; ++k) {
            fbs[k] = 0u;
            if (sm.has(k)) {
                // Position on the coarse axis, held inside the axis (a carried map may not cover this unit's extremes:
                // weights beyond either end all go to the first / last bin, which keeps the map monotone).
                // bin = first bin of the interval + fraction of the interval x bins of the interval, in one fused
                // multiply-add: monotone in w, and at most the first bin of the next interval (the last clamp cannot
                // bind while the table is consistent; it keeps the index inside the counters)
                const float x = fminf(fmaxf(coarse_pos(bin_weight<SPREAD>(key[k], map, stab), lo, scale), 0.0f), (float)COARSE_N - 0.0001f);
                // (a carried map may promise clear low bits that this unit does not have: it then sorts by the network)
                if (SPREAD && ((uint32_t)(key[k] >> 32) & map.lowmask)) smax = (uint32_t)BIN_MAX_KEYS3;
                const uint32_t cb = (uint32_t)(int)x;
                const float fr = __builtin_amdgcn_fractf(x);
                const float2 tb = table[cb];
                const uint32_t fb = min((uint32_t)fmaf(fr, tb.y, tb.x), (uint32_t)(nbins - 1));
                const uint32_t hw = padded ? bin_halfword(fb) : fb;
                const uint32_t sh = (hw & 1u) << 4;
                const uint32_t old = atomicAdd(&hist[hw >> 1], 1u << sh);
                const uint32_t slot = (old >> sh) & 0xFFFFu;
                smax = max(smax, slot);
                fbs[k] = hw | (slot << 16);
            }
        }
    };
    if (__builtin_expect(map.lowmask != 0u, 0)) count_keys(std::true_type{});
    else count_keys(std::false_type{});
    prefetch(1);
    __syncthreads();
    // ---- first rank of every bin: exclusive scan of the counters, written over them (16 bits each)
    bool third_pass = false;      // (the same in every thread)
    {
        const int nq = bpt >> 3;                       // 16-byte pieces of this thread's block
        uint4 *mine = (uint4 *)(hist + tid * hstride);
        uint32_t run = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (q < nq) {
                const uint4 c = mine[q];
                run += (c.x & 0xFFFFu) + (c.x >> 16) + (c.y & 0xFFFFu) + (c.y >> 16) + (c.z & 0xFFFFu) + (c.z >> 16) +
                       (c.w & 0xFFFFu) + (c.w >> 16);
            }
        }
        const uint32_t inc = wave_scan_incl(run);
        const bool wave_over = __ballot(smax >= (uint32_t)BIN_MAX_KEYS) != 0;
        const bool wave_over3 = __ballot(smax >= (uint32_t)BIN_MAX_KEYS3) != 0;
        // one word per wavefront: keys up to and including this wavefront's bins << 3 | a bin too full for three
        // passes << 2 | a bin too full for two << 1 | mass
        if (lane == 63) wtot[wave] = (inc << 3) | (wave_over3 ? 4u : 0u) | (wave_over ? 2u : 0u) | (wave_mass ? 1u : 0u);
        __syncthreads();
        uint32_t below = 0, flags = 0;
        {
            const uint4 *t4 = (const uint4 *)wtot;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint4 t = t4[q];
                const uint32_t e[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (4 * q + i < nw) flags |= e[i];
                    if (4 * q + i < wave) below += e[i] >> 3;
                }
            }
        }
        anymass = (int)(flags & 1u);
        // a bin with more than BIN_MAX_KEYS3 keys anywhere in the unit: the caller sorts by the network instead
        if (flags & 4u) {
            map.have = false;
            return false;
        }
        third_pass = (flags & 2u) != 0u;
        // the counters are read once more (cheaper than carrying them in registers across the barrier)
        uint32_t at = inc - run + below;
        auto step = [&](uint32_t c) -> uint32_t {
            const uint32_t s0 = at;
            at += c & 0xFFFFu;
            const uint32_t s1 = at;
            at += c >> 16;
            return s0 | (s1 << 16);
        };
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (q < nq) {
                uint4 c = mine[q];
                c.x = step(c.x);
                c.y = step(c.y);
                c.z = step(c.z);
                c.w = step(c.w);
                mine[q] = c;
            }
        }
    }
    prefetch(2);
    __syncthreads();
    // ---- scatter: rank = first rank of the bin + slot in the bin
    double *lds = (double *)smem;
    const unsigned short *first = (const unsigned short *)hist;
    const bool unit_weights = !anymass && prm.nseg == 1;
    if (!unit_weights && sm.has(NS - 1)) {
        // every slot holds a key: all first ranks are read before the first key is stored
        uint32_t pos[NS];
#pragma unroll
        for (int k = 0; k < NS; ++k) pos[k] = first[fbs[k] & 0xFFFFu];
#pragma unroll
        for (int k = 0; k < NS; ++k) {
            const uint32_t at = min(pos[k] + (fbs[k] >> 16), (uint32_t)(m - 1));
            lds[swz(at)] = __longlong_as_double((long long)key[k]);
        }
    } else if (!unit_weights) {
#pragma unroll
        for (int k = 0; k < NS; ++k) {
            if (sm.has(k)) {
                // (the clamp cannot bind when the counts are right; it keeps the store inside the row regardless)
                const uint32_t pos = min((uint32_t)first[fbs[k] & 0xFFFFu] + (fbs[k] >> 16), (uint32_t)(m - 1));
                lds[swz(pos)] = __longlong_as_double((long long)key[k]);
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < NS; ++k) {
            if (sm.has(k)) {
                const uint32_t pos = min((uint32_t)first[fbs[k] & 0xFFFFu] + (fbs[k] >> 16), (uint32_t)(m - 1));
                lds[swz(pos)] = __longlong_as_double((long long)unit_weight_key(key[k]));
            }
        }
    }
    prefetch(3);
    __syncthreads();
    // ---- order inside the bins
    const int p0 = tid * EPT;
    const double pad = __longlong_as_double((long long)PAD_KEY);
    double v[EPT];
    if (p0 + EPT <= m) {                 // a whole window: no tests per key
        double *win = lds + swz((uint32_t)p0);
#pragma unroll
        for (int r = 0; r < EPT; ++r) v[r] = win[r];
        sort16(v);
#pragma unroll
        for (int r = 0; r < 8; ++r) win[r] = v[r];
    } else if (p0 < m) {
        const double *src = lds + swz((uint32_t)p0);
#pragma unroll
        for (int r = 0; r < EPT; ++r) v[r] = (p0 + r < m) ? src[r] : pad;
        sort16(v);
        double *dst = lds + swz((uint32_t)p0);
#pragma unroll
        for (int r = 0; r < 8; ++r)
            if (p0 + r < m) dst[r] = v[r];
    }
    // ---- the table for the next unit, from this unit's exact counts: the keys of a coarse interval are the
    // difference of the first ranks of its first bin and of the next interval's first bin.  One wavefront (the
    // last: it has the least to do in the passes) writes it; nothing reads the table before the next unit.
    if (wave == nw - 1) {
        const float4 e0 = ((const float4 *)table)[2 * lane], e1 = ((const float4 *)table)[2 * lane + 1];
        const uint32_t f0 = first[bin_halfword(min((uint32_t)e0.x, (uint32_t)(nbins - 1)))];
        const uint32_t f1 = first[bin_halfword(min((uint32_t)e0.z, (uint32_t)(nbins - 1)))];
        const uint32_t f2 = first[bin_halfword(min((uint32_t)e1.x, (uint32_t)(nbins - 1)))];
        const uint32_t f3 = first[bin_halfword(min((uint32_t)e1.z, (uint32_t)(nbins - 1)))];
        uint32_t f4 = (uint32_t)lane_above((int)f0);
        if (lane == 63) f4 = (uint32_t)m;
        float c[4];
        c[0] = (float)(int)(f1 - f0);
        c[1] = (float)(int)(f2 - f1);
        c[2] = (float)(int)(f3 - f2);
        c[3] = (float)(int)(f4 - f3);
        write_bin_table(table, lane, c, (float)(nbins - COARSE_N - 16) / (4.0f * (float)m));
    }
    __syncthreads();
    // the fine counters start the next unit at zero
    {
        uint4 *hz = (uint4 *)(hist + tid * hstride);
        for (int q = 0; q < (bpt >> 3); ++q) hz[q] = make_uint4(0u, 0u, 0u, 0u);
    }
    if (p0 + EPT + 8 <= m) {
        // upper half of this window (still in registers) with the lower half of the next one, all inside the unit
        double *dst = lds + swz((uint32_t)p0);
        double *dn = lds + swz((uint32_t)(p0 + EPT));
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            v[r] = v[8 + r];
            v[8 + r] = dn[r];
        }
        merge8x8(v);
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            dst[8 + r] = v[r];
            dn[r] = v[8 + r];
        }
    } else if (p0 + 8 < m) {
        const double *nxt = lds + swz((uint32_t)(p0 + EPT));
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            v[r] = v[8 + r];
            v[8 + r] = (p0 + EPT + r < m) ? nxt[r] : pad;
        }
        merge8x8(v);
        double *dst = lds + swz((uint32_t)p0);
        double *dn = lds + swz((uint32_t)(p0 + EPT));
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (p0 + 8 + r < m) dst[8 + r] = v[r];
            if (p0 + EPT + r < m) dn[r] = v[8 + r];
        }
    }
    __syncthreads();
    if (__builtin_expect(third_pass, 0)) {
        // some bin holds 10 to 17 keys: both halves of every window are in order now, merge them
        if (p0 < m) {
            double *win = lds + swz((uint32_t)p0);
#pragma unroll
            for (int r = 0; r < EPT; ++r) v[r] = (p0 + r < m) ? win[r] : pad;
            merge8x8(v);
#pragma unroll
            for (int r = 0; r < EPT; ++r)
                if (p0 + r < m) win[r] = v[r];
        }
        __syncthreads();
    }
    map.have = true;
    return true;
}

// ---------------------------------------------------------------------------------------------
// Kernel 1: load + scale + encode, bitonic sort in LDS, sums, write-out.
// ---------------------------------------------------------------------------------------------
// The 16 W and 16 S values a thread contributes to one unit of work (a row, or one segment of a long row).
// live == false: nothing is read and every slot becomes 0 (the caller has no further unit; assigning all
// slots either way keeps the registers from being carried around the caller's loop).
// part: -1 = all of the unit; 0..3 = the 16-byte loads g with g % 4 == part (VEC), or everything in part 0 (!VEC).
template <int NS, bool VEC>
__device__ __forceinline__ void fetch_unit(const ClusterParams &prm, long long work, int tid, int nth, float (&pw)[NS],
                                           float (&ps)[NS], bool live = true, int part = -1) {
    // (a row has one segment or two: no 64-bit division)
    const long long frow = prm.nseg > 1 ? (work >> 1) : work;
    const int fcol0 = prm.nseg > 1 ? (int)(work & 1) * prm.seglen : 0;
    const int fm = live ? min(prm.m - fcol0, prm.seglen) : 0;
    const Slots<VEC> sm(fm, nth, tid);
    if constexpr (VEC) {
        static_assert(NS % 4 == 0, "16-byte loads fill four slots at a time");
        const float4 *W4 = (const float4 *)(prm.W + frow * prm.ld + fcol0) + tid;
        const float4 *S4 = (const float4 *)(prm.S + frow * prm.ld + fcol0) + tid;
#pragma unroll
        for (int g = 0; g < NS / 4; ++g) {
            if (part >= 0 && (g & 3) != part) continue;
            const bool h = sm.has(4 * g);
            const float4 a = h ? W4[g * nth] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            const float4 b = h ? S4[g * nth] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            pw[4 * g] = a.x; pw[4 * g + 1] = a.y; pw[4 * g + 2] = a.z; pw[4 * g + 3] = a.w;
            ps[4 * g] = b.x; ps[4 * g + 1] = b.y; ps[4 * g + 2] = b.z; ps[4 * g + 3] = b.w;
        }
    } else {
        if (part > 0) return;
        const float *Wr = prm.W + frow * prm.ld + fcol0 + tid;
        const float *Sr = prm.S + frow * prm.ld + fcol0 + tid;
#pragma unroll
        for (int k = 0; k < NS; ++k) {
            const bool h = sm.has(k);
            pw[k] = h ? Wr[k * nth] : 0.0f;
            ps[k] = h ? Sr[k * nth] : 0.0f;
        }
    }
}

// Scaling and key encoding of the values a thread fetched (column tid + k * nth in slot k; padding beyond m).
template <int NS, bool VEC>
__device__ __forceinline__ void build_keys(const float (&pw)[NS], const float (&ps)[NS], const float *alpha, int tid,
                                           int nth, int m, u64 (&key)[NS], bool &mass) {
    const Slots<VEC> sm(m, nth, tid);
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        key[k] = PAD_KEY;
        if (sm.has(k)) {
            float wt, st;
            scaled_pair(pw[k], ps[k], alpha, sm.col(k), wt, st);
            key[k] = make_key(wt, st);
            mass = mass || (st != 0.0f);
        }
    }
}

// NS: key slots per thread, at least ceil(seglen / blockDim.x).  VEC: 16-byte loads of W and S (rows and units
// start at multiples of 16 bytes, lengths are multiples of 4); see Slots for the slot <-> column map.
template <int NS, bool VEC>
__global__ void __launch_bounds__(1024) sort_kernel(ClusterParams prm) {
    extern __shared__ __align__(16) unsigned char smem[];
    u64 *sorted = (u64 *)smem;

    const int tid0 = threadIdx.x, nth = blockDim.x;      // a power of two, at least P / 16

    // A workgroup takes the units of work blockIdx.x, blockIdx.x + gridDim.x, ...  The W and S values
    // of the next unit are fetched into registers (all loads in flight at once) as soon as those of
    // the current unit have been encoded, so that the whole sort of the current unit hides their HBM
    // latency (a long row fills the LDS of a compute unit: no second workgroup is resident to overlap with).
    float pw[NS], ps[NS];
    if ((long long)blockIdx.x < prm.nwork) fetch_unit<NS, VEC>(prm, blockIdx.x, tid0, nth, pw, ps);

    BinMap map;
    map.have = false;
    map.lo = 0.0f;
    map.scale = 0.0f;
    map.lowmask = 0u;
    map.sbm = 0u;
    // Units of work: a workgroup's first two are blockIdx.x and blockIdx.x + gridDim.x; every further one is
    // claimed from a counter in global memory, one unit ahead of the prefetch (the claim for the unit after next
    // is issued while the current unit is sorted, and passes through one LDS word at a barrier the sort has
    // anyway).  A unit that has to take the bitonic network costs about three units of the bucket path: with
    // fixed shares the workgroups that meet such units would finish last and the kernel with them.
    __shared__ int next_slot[2];   // the answers of consecutive units alternate between the two words
    const int nwork = (int)prm.nwork;
    if (tid0 == 0) next_slot[0] = (int)min((long long)blockIdx.x + gridDim.x, prm.nwork);
    __syncthreads();
    int next = 0, par = 0;
    for (int work = (int)blockIdx.x; work < nwork; work = next, par ^= 1) {
    // the unit that is fetched while this one is sorted: the answer to the previous unit's claim
    next = prm.bk_bpt > 0 ? __builtin_amdgcn_readfirstlane(next_slot[par]) : (int)min((long long)work + gridDim.x, prm.nwork);
    // the thread index is made opaque per unit: per-thread addresses are recomputed where they are
    // used instead of being hoisted out of this loop and held in registers through the sort
    int tid = tid0;
    asm volatile("" : "+v"(tid));
    const long long row = prm.nseg > 1 ? (work >> 1) : work;
    const int col0 = prm.nseg > 1 ? (int)(work & 1) * prm.seglen : 0;   // first column of this segment
    const int m = min(prm.m - col0, prm.seglen);                     // keys sorted by this workgroup
    const float *alpha = prm.alpha ? prm.alpha + col0 : nullptr;
    const bool more = next < nwork;
    const bool buckets = prm.bk_bpt > 0;
    const Slots<VEC> sm(m, nth, tid);

    // keys in registers, and whether the unit holds any sensitivity mass
    u64 key[NS];
    bool mass = false;
    build_keys<NS, VEC>(pw, ps, alpha, tid, nth, m, key, mass);
    // (the bitonic network needs the registers: without the bucket path the next unit is fetched after the sort)
    // the claim for the unit after next: thread 0 asks, and puts the answer into the other word of next_slot ahead
    // of one of the unit's barriers; everybody reads it at the start of the next unit (this unit's word is
    // written again two units on, behind barriers every reader has passed by then)
    unsigned claim = 0u;
    auto claim_next = [&]() {
        if (more && tid == 0) claim = (unsigned)atomicAdd(prm.work_counters, 1);
    };
    auto publish = [&]() {
        if (tid == 0) next_slot[par ^ 1] = more ? (int)min(2ll * gridDim.x + (long long)claim, (long long)nwork) : nwork;
    };
    auto prefetch = [&](int part) {
        fetch_unit<NS, VEC>(prm, more ? next : work, tid, nth, pw, ps, more, part);
        if (part == 1) publish();
    };
    if (buckets) {
        claim_next();
        prefetch(0);
    }
    int anymass = 1;
    bool sorted_ok = false;
    if (buckets) {
        const bool wave_mass = __ballot(mass) != 0;
        bool usable = true;
        if (__builtin_expect(!map.have, 0)) {
            // no map carried over: the axis is this unit's own range.  Per wavefront: least and largest weight and
            // the mass flag, for everybody after the barrier below
            float *wmin = (float *)(smem + prm.bk_misc_off + BK_WMIN), *wmax = (float *)(smem + prm.bk_misc_off + BK_WMAX);
            uint32_t *wmass = (uint32_t *)(smem + prm.bk_misc_off + BK_WMASS);
            {
                float wlo = INFINITY, whi = -INFINITY;
#pragma unroll
                for (int k = 0; k < NS; ++k) {
                    if (sm.has(k)) {
                        wlo = fminf(wlo, elem_w(key[k]));
                        whi = fmaxf(whi, elem_w(key[k]));
                    }
                }
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) {
                    wlo = fminf(wlo, __shfl_xor(wlo, o, 64));
                    whi = fmaxf(whi, __shfl_xor(whi, o, 64));
                }
                if ((tid & 63) == 0) {
                    wmin[tid >> 6] = wlo;
                    wmax[tid >> 6] = whi;
                    wmass[tid >> 6] = wave_mass ? 1u : 0u;
                }
            }
            uint32_t *cc = (uint32_t *)(smem + prm.bk_coarse_off);
            for (int i = tid; i < COARSE_N * 4; i += nth) cc[i] = 0u;
            // which bits any weight of the unit has set, and the typical exponent of s (sum and count of the
            // exponent fields of the positive s)
            uint32_t *wor = (uint32_t *)(smem + prm.bk_misc_off + BK_WOR);
            uint32_t *sex = (uint32_t *)(smem + prm.bk_misc_off + BK_SMIN), *scn = (uint32_t *)(smem + prm.bk_misc_off + BK_SMAX);
            {
                uint32_t orb = 0u, esum = 0u, ecnt = 0u;
#pragma unroll
                for (int k = 0; k < NS; ++k) {
                    if (sm.has(k)) {
                        const uint32_t h = (uint32_t)(key[k] >> 32), l = (uint32_t)key[k];
                        const uint32_t sb = (h >> 31) ? ~l : l;
                        orb |= h;
                        esum += sb >> 23;
                        ecnt += sb ? 1u : 0u;
                    }
                }
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) {
                    orb |= (uint32_t)__shfl_xor((int)orb, o, 64);
                    esum += (uint32_t)__shfl_xor((int)esum, o, 64);
                    ecnt += (uint32_t)__shfl_xor((int)ecnt, o, 64);
                }
                if ((tid & 63) == 0) {
                    wor[tid >> 6] = orb;
                    sex[tid >> 6] = esum;
                    scn[tid >> 6] = ecnt;
                }
            }
            __syncthreads();
            const int nw = nth >> 6;
            float lo = INFINITY, hi = -INFINITY;
            uint32_t any = 0;
            {
                uint32_t orb = 0u, esum = 0u, ecnt = 0u;
                for (int w2 = 0; w2 < nw; ++w2) {
                    orb |= wor[w2];
                    esum += sex[w2];
                    ecnt += scn[w2];
                }
                // clear low bits of the mantissa only (a row of zeros and powers of two would clear more), 16 at
                // most; fewer than 8 leave the values distinct enough
                int kz = orb ? min(__builtin_ctz(orb), 16) : 0;
                if (kz < 8) kz = 0;
                const int emean = ecnt ? (int)(esum / ecnt) : 127;
                // (the same in every lane: kept in scalar registers)
                map.lowmask = (uint32_t)__builtin_amdgcn_readfirstlane((int)((1u << kz) - 1u));
                map.sbm = (uint32_t)__builtin_amdgcn_readfirstlane((int)(((uint32_t)emean << 23) + (1u << 22)));
            }
            if (map.lowmask) {
                // the fill table: counts of s per piece (16 copies of the counters, in the space of the value
                // bins' counters, which are cleared again below), running sums scaled to the fill values
                uint32_t *sh = (uint32_t *)(smem + prm.bk_hist_off);
                uint32_t *stabw = (uint32_t *)(smem + prm.bk_misc_off + BK_STAB);
                for (int i = tid; i < STAB_N * 16; i += nth) sh[i] = 0u;
                __syncthreads();
#pragma unroll
                for (int k = 0; k < NS; ++k) {
                    if (sm.has(k)) {
                        const uint32_t h = (uint32_t)(key[k] >> 32), l = (uint32_t)key[k];
                        int idx;
                        uint32_t f16;
                        fill_piece((h >> 31) ? ~l : l, map.sbm, idx, f16);
                        atomicAdd(&sh[idx * 16 + (tid & 15)], 1u);
                    }
                }
                __syncthreads();
                if (tid < 64) {
                    uint32_t c = 0u;
                    for (int q = 0; q < 16; ++q) c += sh[tid * 16 + q];
                    const uint32_t inc = wave_scan_incl(c);
                    // share of the keys below piece tid, in fill values (m <= 32768, the mask <= 65535: no overflow)
                    stabw[tid] = (uint32_t)(((unsigned long long)(inc - c) * (map.lowmask + 1u)) / (uint32_t)m);
                    if (tid == 63) stabw[64] = map.lowmask + 1u;
                }
                __syncthreads();
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 a = ((const float4 *)wmin)[q], b4 = ((const float4 *)wmax)[q];
                const uint4 c = ((const uint4 *)wmass)[q];
                if (4 * q + 0 < nw) { lo = fminf(lo, a.x); hi = fmaxf(hi, b4.x); any |= c.x; }
                if (4 * q + 1 < nw) { lo = fminf(lo, a.y); hi = fmaxf(hi, b4.y); any |= c.y; }
                if (4 * q + 2 < nw) { lo = fminf(lo, a.z); hi = fmaxf(hi, b4.z); any |= c.z; }
                if (4 * q + 3 < nw) { lo = fminf(lo, a.w); hi = fmaxf(hi, b4.w); any |= c.w; }
            }
            anymass = (int)any;
            // a usable axis needs two distinct finite ends (a constant row has none);
            // (1 - 2^-20): the largest weight stays below the end of the axis
            usable = hi > lo && (hi - lo) < INFINITY;
            map.lo = lo;
            map.scale = (float)COARSE_N / (hi - lo) * 0.99999904632568359375f;
        }
        if (usable) sorted_ok = bucket_sort<NS, VEC>(smem, prm, key, tid, nth, m, map, wave_mass, anymass, prefetch);
        else publish();
    } else {
        anymass = __syncthreads_or((int)mass);
    }
    // (a segment of a long row cannot tell on its own: it records what it saw for merge_tile_kernel)
    if (prm.nseg > 1 && tid == 0) prm.segmass[work] = anymass;
    if (!sorted_ok) {      // (no branch hint here: with one the compiler runs the 12-slot variant out of registers)
        // The bitonic network over the whole padded row.  Its keys overlay the bucket path's tables: wait
        // until every thread is done with them.  The bucket path gave its key registers away, so the
        // unit is read and encoded once more, and the next unit fetched again after it (rare).
        if (buckets) {
            __syncthreads();
            fetch_unit<NS, VEC>(prm, work, tid, nth, pw, ps);
            bool mass2 = false;
            build_keys<NS, VEC>(pw, ps, alpha, tid, nth, m, key, mass2);
        }
        if (!anymass && prm.nseg == 1) {
            // no sensitivity mass in this row: cluster with unit weights
#pragma unroll
            for (int k = 0; k < NS; ++k)
                if (sm.has(k)) key[k] = unit_weight_key(key[k]);
        }
#pragma unroll
        for (int k = 0; k < NS; ++k)
            if (sm.col(k) < prm.P) sorted[swz((uint32_t)sm.col(k))] = key[k];
        for (int j = tid + NS * nth; j < prm.P; j += nth) sorted[swz((uint32_t)j)] = PAD_KEY;   // padding no slot covers
        __syncthreads();
        // (the variants with 16-byte loads serve fixed ranges of the padded length: 8 slots up to 8192 keys, 12 and
        // 16 slots 16384; only the networks a variant can be asked for are compiled into it)
        if constexpr (VEC && NS > 8) {
            sort_row<14>((double *)sorted, (uint32_t)tid, m);
        } else {
            switch (prm.logP) {
                case 10: sort_row<10>((double *)sorted, (uint32_t)tid, m); break;
                case 11: sort_row<11>((double *)sorted, (uint32_t)tid, m); break;
                case 12: sort_row<12>((double *)sorted, (uint32_t)tid, m); break;
                case 13: sort_row<13>((double *)sorted, (uint32_t)tid, m); break;
                default:
                    if constexpr (!VEC) sort_row<14>((double *)sorted, (uint32_t)tid, m);
                    break;
            }
        }
        fetch_unit<NS, VEC>(prm, more ? next : work, tid, nth, pw, ps, more);
    }

    if (prm.nseg > 1) {
        // one segment of a long row: sorted keys only; merge_tile_kernel does the rest
        u64 *kseg = prm.keys_seg + row * (long long)prm.m + col0;
        for (int j = tid; j < m; j += nth) kseg[j] = sorted[swz((uint32_t)j)];
        if (!buckets) __syncthreads();   // the LDS is refilled for the next unit (see the end of the loop)
        continue;
    }
    // sums of s and s*w over each 16-key chunk (s*w of two floats is exact in float64), the weight
    // of the chunk's first key, and the sums over each group of 4 chunks (4 neighbouring threads)
    {
        const bool mine_ok = tid * EPT < m;
        const u64 *mine = sorted + swz((uint32_t)(mine_ok ? tid * EPT : 0));
        double c = 0.0, q = 0.0, r2 = 0.0;
        float w0 = 0.0f;
        auto add_key = [&](u64 el, int e) {
            const double sv = (double)elem_s(el), wv = (double)elem_w(el);
            if (e == 0) w0 = elem_w(el);
            c += sv;
            q = fma(sv, wv, q);
            r2 = fma(sv * wv, wv, r2);     // second moment, for the row errors
        };
        if (tid * EPT + EPT <= m) {        // a whole chunk: no tests per key
#pragma unroll
            for (int e = 0; e < EPT; ++e) add_key(mine[e], e);
        } else {
#pragma unroll
            for (int e = 0; e < EPT; ++e) add_key((tid * EPT + e < m) ? mine[e] : NEUTRAL_KEY, e);
        }
        if (mine_ok) {
            prm.L1[row * prm.n1 + tid] = make_double2(c, q);
            prm.R1[row * prm.n1 + tid] = r2;
            prm.w16[row * prm.n1 + tid] = w0;
        }
        const double c4 = quad_sum(c), q4 = quad_sum(q), r4 = quad_sum(r2);   // threads past the row add zeros
        if (mine_ok && (tid & 3) == 0) {
            prm.Q[row * prm.nq + (tid >> 2)] = make_double2(c4, q4);
            prm.RQ[row * prm.nq + (tid >> 2)] = r4;
        }
    }
    // sorted keys, compact and in rank order
    u64 *keys = prm.keys + row * (long long)m;
    for (int j = tid; j < m; j += nth) keys[j] = plain_key(sorted[swz((uint32_t)j)]);
    // The next unit refills the key region of the LDS.  On the bucket path it first works on its tables, which
    // lie beyond that region, and passes several barriers before its scatter; its bitonic branch has a barrier
    // of its own.  Without the bucket path the refill is immediate.
    if (!buckets) __syncthreads();
    }
    // the last workgroup to get here leaves both counters at zero for the next launch (every claim of every
    // workgroup has been answered by then: a workgroup uses the answers before it leaves its loop)
    if (tid0 == 0) {
        const int done = atomicAdd(prm.work_counters + 1, 1);
        if (done == (int)gridDim.x - 1) {
            atomicExch(prm.work_counters, 0);
            atomicExch(prm.work_counters + 1, 0);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Rows longer than one LDS sort (m > 16384): the two sorted segments A, B of a row are merged tile by tile.
// A workgroup produces MG_TILE consecutive keys of the merged row: two wavefronts find, by a 64-way
// search in global memory, how many keys of A lie ahead of the tile's first and last output (merge path,
// equal keys from A first); the keys in between, MG_TILE in all, are staged in LDS; every thread then
// finds the split for its own 16 outputs by binary search in LDS, loads its share of A ascending and of B
// descending (a bitonic sequence) and sorts it with the 4-stage merge network in registers.  The 16 outputs
// are one chunk: its sums, and with the neighbours' the sums of 4 chunks, are written with the keys (the
// quantities sort_kernel produces for short rows).  A row without sensitivity mass in either segment gets
// unit weights here.
// ---------------------------------------------------------------------------------------------
constexpr int MG_THREADS = 256;
constexpr int MG_TILE = MG_THREADS * EPT;

// Number of keys of A among the first o keys of merge(A, B), equal keys from A first.  The predicate
// p(x) = A[x] <= B[o-1-x] holds exactly for x below the answer; 64 lanes probe 64 positions per round.
__device__ __forceinline__ int merge_split_wave(const double *__restrict__ A, int la, const double *__restrict__ B,
                                                int lb, int o, int lane) {
    int lo = max(0, o - lb), hi = min(o, la);
    while (hi > lo) {
        const int step = (hi - lo + 63) >> 6;
        const int x = lo + lane * step;
        const bool p = (x < hi) && (A[x] <= B[o - 1 - x]);
        const int nt = __popcll(__ballot(p));          // probes 0 .. nt-1 are true
        const int nlo = nt > 0 ? lo + (nt - 1) * step + 1 : lo;
        hi = min(hi, lo + nt * step);
        lo = nlo;
    }
    return lo;
}

__global__ void __launch_bounds__(MG_THREADS) merge_tile_kernel(ClusterParams prm, int tiles_per_row) {
    __shared__ double buf[MG_TILE + MG_TILE / 16];
    __shared__ int part[MG_THREADS + 1];
    __shared__ int split[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long row = blockIdx.x / tiles_per_row;
    const int tile = (int)(blockIdx.x % tiles_per_row);
    const int m = prm.m;
    const int la = min(prm.seglen, m), lb = m - la;
    const double *__restrict__ A = (const double *)(prm.keys_seg + row * (long long)m);
    const double *__restrict__ B = A + la;
    const int o0 = tile * MG_TILE, o1 = min(m, o0 + MG_TILE);
    const int T = o1 - o0;
    if (wave < 2) {
        const int sp = merge_split_wave(A, la, B, lb, wave == 0 ? o0 : o1, lane);
        if (lane == 0) split[wave] = sp;
    }
    __syncthreads();
    const int ia0 = split[0], ia1 = split[1];
    const int ib0 = o0 - ia0;
    const int lat = ia1 - ia0, lbt = T - lat;            // keys of A and of B in this tile
    for (int x = tid; x < T; x += MG_THREADS)
        buf[swz((uint32_t)x)] = x < lat ? A[ia0 + x] : B[ib0 + (x - lat)];
    __syncthreads();
    // this thread's outputs: d .. d + cnt - 1 of the tile
    const int d = tid * EPT;
    const int cnt = max(0, min(EPT, T - d));
    int i = lat;                                          // keys of A ahead of output d
    if (d < T) {
        int lo = max(0, d - lbt), hi = min(d, lat);
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (buf[swz((uint32_t)mid)] <= buf[swz((uint32_t)(lat + d - 1 - mid))]) lo = mid + 1;
            else hi = mid;
        }
        i = lo;
    }
    part[tid] = i;
    if (tid == 0) part[MG_THREADS] = lat;
    __syncthreads();
    const int acnt = (d < T) ? ((d + EPT >= T) ? lat - i : part[tid + 1] - i) : 0;
    const int bcnt = cnt - acnt;
    const int jb = d - i;                                 // keys of B ahead of output d
    const double inf = __longlong_as_double((long long)PAD_KEY);
    double v[EPT];
#pragma unroll
    for (int r = 0; r < EPT; ++r) {
        const bool fromA = r < acnt, fromB = r >= EPT - bcnt;
        const int idx = fromA ? i + r : lat + jb + (EPT - 1 - r);
        v[r] = (fromA || fromB) ? buf[swz((uint32_t)idx)] : inf;
    }
#pragma unroll
    for (int rb = 3; rb >= 0; --rb) {
#pragma unroll
        for (int r = 0; r < EPT; ++r)
            if (!(r & (1 << rb))) ce(v[r], v[r | (1 << rb)]);
    }
    const bool unit = (prm.segmass[row * 2] | prm.segmass[row * 2 + 1]) == 0;
    // the merged keys go back to LDS (every thread has read what it needs: barrier) and from there to global
    // memory with consecutive lanes on consecutive keys (16 keys per thread written in place would put the 64
    // lanes of a store on 64 different lines)
    __syncthreads();
    u64 *obuf = (u64 *)buf;
    double c = 0.0, q = 0.0, r2 = 0.0;
    float w0 = 0.0f;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        u64 el = NEUTRAL_KEY;
        if (e < cnt) {
            el = (u64)__double_as_longlong(v[e]);
            if (unit) el = unit_weight_key(el);
            obuf[swz((uint32_t)(d + e))] = plain_key(el);
        }
        const double sv = (double)elem_s(el), wv = (double)elem_w(el);
        if (e == 0) w0 = elem_w(el);
        c += sv;
        q = fma(sv, wv, q);
        r2 = fma(sv * wv, wv, r2);
    }
    const long long ch = (long long)(o0 + d) >> 4;
    if (cnt > 0) {
        prm.L1[row * prm.n1 + ch] = make_double2(c, q);
        prm.R1[row * prm.n1 + ch] = r2;
        prm.w16[row * prm.n1 + ch] = w0;
    }
    const double c4 = quad_sum(c), q4 = quad_sum(q), r4 = quad_sum(r2);   // threads past the row add zeros
    if (cnt > 0 && (tid & 3) == 0) {
        prm.Q[row * prm.nq + (ch >> 2)] = make_double2(c4, q4);
        prm.RQ[row * prm.nq + (ch >> 2)] = r4;
    }
    __syncthreads();
    u64 *keys = prm.keys + row * (long long)m + o0;
    for (int x = tid; x < T; x += MG_THREADS) keys[x] = obuf[swz((uint32_t)x)];
}

// ---------------------------------------------------------------------------------------------
// Kernel 2: Lloyd iterations.
// ---------------------------------------------------------------------------------------------

// Sums over whole 16-key chunks.  Level 0 = chunk sums (global memory, written by the sort); level 1 = groups of
// 4 chunks (64 keys).  For sum s and sum s*w a workgroup keeps, per row, the running sums ahead of every group in
// LDS as double-double numbers (an unevaluated pair hi + lo, about 106 bits): the sum over a range of groups is the
// difference of two of them, exact to about 2^-104 of the row total, so a cluster of tiny mass next to a heavy
// element keeps full relative precision (a difference of plain float64 running sums would not).  The second
// moments (sum s*w*w), needed once at the end, form a radix-4 tree: level 1 in global memory, levels >= 2 in LDS.
struct LevelMap {
    int nlev;        // levels 0 .. nlev-1 of the second-moment tree
    int n[8];        // entries per level
    int roff[8];     // byte offset of the second-moment sums of level >= 2 inside the row's LDS block
    int w16_off, ppd_off, ppn_off, bytes;   // first weights; running sums of s and of s*w (n[1] + 1 double2 each)
};
__host__ __device__ inline LevelMap level_map(int n1u) {
    LevelMap L;
    L.w16_off = 0;
    int o = (n1u * 4 + 15) & ~15;
    L.n[0] = n1u;
    int lv = 0, n = n1u;
    do {
        n = (n + 3) >> 2;
        ++lv;
        L.n[lv] = n;
    } while (n > 1);
    for (int k = lv + 1; k < 8; ++k) L.n[k] = 0;
    L.nlev = lv + 1;
    L.ppd_off = o;
    o += (L.n[1] + 1) * 16;
    L.ppn_off = o;
    o += (L.n[1] + 1) * 16;
    L.roff[0] = 0;
    L.roff[1] = 0;
    for (int k = 2; k < 8; ++k) {
        L.roff[k] = o;
        o += ((L.n[k] * 8) + 15) & ~15;
    }
    L.bytes = o;
    return L;
}

// Double-double arithmetic on (hi, lo) pairs held in a double2 (x = hi, y = lo).
__device__ __forceinline__ double2 dd_add(double2 a, double2 b) {
    const double s = a.x + b.x;
    const double bb = s - a.x;
    double e = (a.x - (s - bb)) + (b.x - bb);     // a.x + b.x = s + e exactly
    e += a.y + b.y;
    const double h = s + e;
    return make_double2(h, e - (h - s));
}
// b - a rounded to one double
__device__ __forceinline__ double dd_diff(double2 b, double2 a) {
    const double s = b.x - a.x;
    const double bb = s - b.x;
    const double e = (b.x - (s - bb)) + (-a.x - bb);   // b.x - a.x = s + e exactly
    return s + (e + (b.y - a.y));
}
// x of the lane selected by a DPP control word in the lanes of the enabled rows, 0 elsewhere and where the
// pattern has no source lane
template <int CTRL, int ROWS>
__device__ __forceinline__ double dpp_or_zero(double x) {
    const long long b = __double_as_longlong(x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)b, CTRL, ROWS, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, ROWS, 0xF, false);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
template <int CTRL, int ROWS>
__device__ __forceinline__ double2 dd_scan_step(double2 x) {
    const double2 t = make_double2(dpp_or_zero<CTRL, ROWS>(x.x), dpp_or_zero<CTRL, ROWS>(x.y));
    return dd_add(x, t);
}
// inclusive double-double prefix sum over the 64 lanes (the pattern of wave_scan_incl)
__device__ __forceinline__ double2 dd_wave_scan_incl(double2 x) {
    x = dd_scan_step<0x111, 0xF>(x);
    x = dd_scan_step<0x112, 0xF>(x);
    x = dd_scan_step<0x114, 0xF>(x);
    x = dd_scan_step<0x118, 0xF>(x);
    x = dd_scan_step<0x142, 0xA>(x);
    x = dd_scan_step<0x143, 0xC>(x);
    return x;
}

constexpr int ITER_THREADS = 64;   // one wavefront serves two rows
constexpr int MAX_LEVELS = 8;

// One lane per cluster.  A row takes 30 lanes of a half wavefront: bit width 1 on lanes 0-1, 2 on
// 2-5, 3 on 6-13, 4 on 14-29 (position p = centroids ordered by value); two rows per wavefront.
// Per iteration a lane finds the lower boundary of its cluster in two steps -- the chunk that
// holds it, by a search over the chunks' first weights in LDS, then the rank inside that chunk
// from its 16 keys (one round of global loads) -- and adds up its range from: the keys of its own
// boundary chunk, the lower part of the next cluster's boundary chunk (handed over by that lane),
// and the whole chunks in between: up to 3 chunk sums at either end (global memory) and the whole groups
// of 4 chunks as a difference of two double-double running sums (LDS).
typedef u64 u64x2 __attribute__((ext_vector_type(2)));
typedef u64x2 __attribute__((aligned(8))) u64x2_a8;

// Quotient n / d for d > 0 within about one unit in the last place (reciprocal estimate, two
// Newton steps, one correction): the centroid update needs no correctly rounded division, its
// operands already carry the rounding of the sums.
__device__ __forceinline__ double quick_div(double n, double d) {
    double r = __builtin_amdgcn_rcp(d);
    r = fma(fma(-d, r, 1.0), r, r);
    r = fma(fma(-d, r, 1.0), r, r);
    const double q = n * r;
    return fma(fma(-d, q, n), r, q);
}

// RAGGED: the row length is not a multiple of 16, so the last chunk holds fewer than 16 keys.
// WAVES: wavefronts per SIMD the kernel is compiled for.  2 needs no spills (187 registers); when a matrix has more
// rows than 2 per SIMD can hold at once, 3 (168 registers, about 70 of them spilled) finishes sooner all the same.
template <bool RAGGED, int WAVES>
__global__ void __launch_bounds__(ITER_THREADS) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES)))
lloyd_iter_kernel(ClusterParams prm, long long nrows, LevelMap LM) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int m = prm.m;
    const int n1u = (m + 15) >> 4;   // LM = level_map(n1u), worked out by the host
    const int lane = threadIdx.x;
    const int h = lane >> 5, l5 = lane & 31;

    // ---- prologue: both rows' first weights, running sums and second-moment levels into LDS -------
    // All that the two rows need first is requested in one go (one trip to global memory instead of one per
    // array and row): the groups' sums, the first 512 first weights, the first 64 level-2 second moments.
    const int nhalf = (2ll * blockIdx.x + 1 < nrows) ? 2 : 1;
    const int ng = LM.n[1];
    const int per = (ng + ITER_THREADS - 1) / ITER_THREADS;     // groups per lane: at most 8 (rows of up to 32768 keys)
    double2 qv[2][8];
    float t8[2][8];
    double rq4[2][4];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        const long long rr = 2ll * blockIdx.x + (hh < nhalf ? hh : 0);
        const double2 *gq = prm.Q + rr * prm.nq;
        const float *gw = prm.w16 + rr * prm.n1;
        const double *grq = prm.RQ + rr * prm.nq;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int q = lane * per + k;
            qv[hh][k] = (k < per && q < ng) ? gq[q] : make_double2(0.0, 0.0);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = u * ITER_THREADS + lane;
            t8[hh][u] = (j < n1u) ? gw[j] : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) rq4[hh][k] = (LM.nlev > 2 && 4 * lane + k < ng) ? grq[4 * lane + k] : 0.0;
    }
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        if (hh >= nhalf) break;
        const long long rr = 2ll * blockIdx.x + hh;
        unsigned char *blkw = smem + (size_t)hh * LM.bytes;
        float *w16w = (float *)(blkw + LM.w16_off);
        const float *gw = prm.w16 + rr * prm.n1;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = u * ITER_THREADS + lane;
            if (j < n1u) w16w[j] = t8[hh][u];
        }
        for (int j0 = 8 * ITER_THREADS; j0 < n1u; j0 += 8 * ITER_THREADS) {
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int j = j0 + u * ITER_THREADS + lane;
                t[u] = (j < n1u) ? gw[j] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int j = j0 + u * ITER_THREADS + lane;
                if (j < n1u) w16w[j] = t[u];
            }
        }
        // running sums ahead of every group of 4 chunks, pp[ng] = row total.  A lane takes `per` consecutive
        // groups; one double-double scan over the lanes per quantity.
        {
            double2 *ppd = (double2 *)(blkw + LM.ppd_off), *ppn = (double2 *)(blkw + LM.ppn_off);
            double2 md = make_double2(0.0, 0.0), mn = make_double2(0.0, 0.0);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                md = dd_add(md, make_double2(qv[hh][k].x, 0.0));
                mn = dd_add(mn, make_double2(qv[hh][k].y, 0.0));
            }
            const double2 id = dd_wave_scan_incl(md), in = dd_wave_scan_incl(mn);
            // sums of the lanes below: the inclusive sums shifted up by one lane
            double2 rd = make_double2(lane_below(id.x), lane_below(id.y));
            double2 rn = make_double2(lane_below(in.x), lane_below(in.y));
            if (lane == 0) {
                rd = make_double2(0.0, 0.0);
                rn = make_double2(0.0, 0.0);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int q = lane * per + k;
                if (k < per && q < ng) {
                    ppd[q] = rd;
                    ppn[q] = rn;
                    rd = dd_add(rd, make_double2(qv[hh][k].x, 0.0));
                    rn = dd_add(rn, make_double2(qv[hh][k].y, 0.0));
                    if (q == ng - 1) {
                        ppd[ng] = rd;
                        ppn[ng] = rn;
                    }
                }
            }
        }
        // second moments: level 2 from the groups' sums in global memory
        if (LM.nlev > 2) {
            const double *grq = prm.RQ + rr * prm.nq;
            double *r2 = (double *)(blkw + LM.roff[2]);
            if (lane < LM.n[2]) r2[lane] = ((rq4[hh][0] + rq4[hh][1]) + rq4[hh][2]) + rq4[hh][3];
            for (int q = lane + ITER_THREADS; q < LM.n[2]; q += ITER_THREADS) {
                double acc = 0.0;
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (4 * q + k < ng) acc += grq[4 * q + k];
                r2[q] = acc;
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int lv = 3; lv < MAX_LEVELS; ++lv) {
        if (lv < LM.nlev) {
            for (int hh = 0; hh < nhalf; ++hh) {
                unsigned char *blkw = smem + (size_t)hh * LM.bytes;
                const double *rsrc = (const double *)(blkw + LM.roff[lv - 1]);
                double *rdst = (double *)(blkw + LM.roff[lv]);
                for (int q = lane; q < LM.n[lv]; q += ITER_THREADS) {
                    double rr2 = 0.0;
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (4 * q + k < LM.n[lv - 1]) rr2 += rsrc[4 * q + k];
                    rdst[q] = rr2;
                }
            }
            __syncthreads();
        }
    }

    // ---- lane -> (row, bit width, position) ------------------------------------------------------
    const long long row = 2ll * blockIdx.x + h;
    const bool rowok = row < nrows;
    int b, p, L0;
    if (l5 < 2) { b = 1; p = l5; L0 = 0; }
    else if (l5 < 6) { b = 2; p = l5 - 2; L0 = 2; }
    else if (l5 < 14) { b = 3; p = l5 - 6; L0 = 6; }
    else if (l5 < 30) { b = 4; p = l5 - 14; L0 = 14; }
    else { b = 0; p = 0; L0 = 30; }
    L0 += 32 * h;
    const int K = 1 << b;
    const long long rowc = rowok ? row : 0;
    const int rowbits = (prm.bits && rowok) ? (int)prm.bits[row] : 0;
    const bool on = rowok && b > 0 && (prm.bits ? (b == rowbits) : (b >= prm.bmin && b <= prm.bmax));
    const u64 maskb = ((1ull << K) - 1ull) << L0;
    auto from_pos = [&](int k) -> int { return min(L0 + k, 63); };   // lane of position k of this bit width

    const unsigned char *blk = smem + (size_t)h * LM.bytes;
    const float *w16 = (const float *)(blk + LM.w16_off);
    const double2 *ppd = (const double2 *)(blk + LM.ppd_off), *ppn = (const double2 *)(blk + LM.ppn_off);
    const u64 *__restrict__ keys = prm.keys + rowc * (long long)m;
    const double2 *__restrict__ L1 = prm.L1 + rowc * prm.n1;

    // ---- weighted-quantile start with strictly increasing ranks ---------------------------------
    int r = 0;
    float wstart = 0.0f;     // weight of the key at rank r, when r ends up inside the chunk read below
    bool wstart_ok = false;
    {
        const double total = ppd[ng].x;
        const double tau = total * (double)(2 * p + 1) / (double)(2 * K);
        // largest group g with pre[g] < tau (pre[0] = 0 < tau)
        int lo = 0, hi = on ? ng - 1 : 0;
        while (__ballot(lo < hi)) {
            const int mid = (lo + hi + 1) >> 1;
            const double x = ppd[min(mid, ng)].x;
            if (lo < hi) {
                if (x < tau) lo = mid; else hi = mid - 1;
            }
        }
        // chunk inside the group: largest chunk whose running sum ahead of it is < tau
        int chunk = 4 * lo;
        double acc = ppd[lo].x;
        u64 el[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) el[j] = NEUTRAL_KEY;
        if (on) {
            double dch[3];
#pragma unroll
            for (int k = 0; k < 3; ++k) dch[k] = (chunk + k + 1 < n1u) ? L1[chunk + k].x : 0.0;
            bool go = true;
            const int c0 = chunk;
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const double nx = acc + dch[k];
                const bool t = go && (c0 + k + 1 < n1u) && (nx < tau);
                if (t) {
                    acc = nx;
                    chunk = c0 + k + 1;
                } else {
                    go = false;
                }
            }
            const int r0 = chunk * 16;
#pragma unroll
            for (int j = 0; j < 16; ++j) el[j] = (r0 + j < m) ? keys[r0 + j] : NEUTRAL_KEY;
            int found = min(r0 + 15, m - 1);
            bool hit = false;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                acc += (double)plain_s(el[j]);
                if (!hit && r0 + j < m && acc >= tau) {
                    found = r0 + j;
                    hit = true;
                }
            }
            r = found;
        }
        int prev = -1;
        for (int k = 0; k < 16; ++k) {
            int rk = __shfl(r, from_pos(k), 64);
            if (k < K) {
                rk = max(rk, prev + 1);
                rk = min(rk, m - K + k);
                if (p == k) r = rk;
                prev = rk;
            }
        }
        if (on) {
            // the repair seldom moves a rank out of the 16 keys already in registers
            const int off = r - chunk * 16;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (off == j) { wstart = elem_w(el[j]); wstart_ok = true; }
        }
    }
    if (__ballot(on && !wstart_ok) != 0) {
        if (on && !wstart_ok) wstart = elem_w(keys[r]);
    }
    double v = on ? (double)wstart : 0.0;
    int idx = p;
    int Bcur = 0, Bold = -1, idxold = -1, cold = 0;
    double Dk = 0.0, Nk = 0.0;       // sums of this lane's cluster under the last assignment it took part in
    bool emptyk = false;             // ... in which it owned nothing (its value repeated the one below)
    bool done = !on;

    // the boundary chunk of the previous iteration stays in registers: late iterations move a boundary by a few
    // ranks, inside the same 16 keys, and then the lane asks the memory system for nothing
    u64 el[16];
    int cl_held = -2;
    for (int it = 0; it < prm.iters; ++it) {
        if (__ballot(!done) == 0) break;
        const bool live = !done;     // this lane's bit width still iterates
        double vlo = lane_below(v);
        int ilo = lane_below(idx);
        {   // keep positions ordered by (value, cluster index)
            const bool ok = done || (p == 0) || (vlo < v) || (vlo == v && ilo < idx);
            if (__builtin_expect(__ballot(!ok) != 0, 0)) {
                int rank = 0;
                for (int k = 0; k < 16; ++k) {
                    const double vq = shfl_d(v, from_pos(k));
                    const int iq = __shfl(idx, from_pos(k), 64);
                    if (k < K) rank += (vq < v || (vq == v && iq < idx)) ? 1 : 0;
                }
                int src = p;
                for (int k = 0; k < 16; ++k) {
                    const int rq = __shfl(rank, from_pos(k), 64);
                    if (k < K && rq == p) src = k;
                }
                const double nv = shfl_d(v, from_pos(src));
                const int ni = __shfl(idx, from_pos(src), 64);
                if (!done) {
                    v = nv;
                    idx = ni;
                }
                vlo = lane_below(v);
                ilo = lane_below(idx);
            }
        }
        const bool dup = !done && (p > 0) && (vlo == v);
        int rep = idx;       // lowest cluster index among the positions sharing this value
        int replo = ilo;
        const bool anydup = __ballot(dup) != 0;
        if (__builtin_expect(anydup, 0)) {
            int rs = p;      // first position of this position's run of equal values
            for (int k = 1; k < 16; ++k) {
                const int dk = __shfl((int)dup, from_pos(k), 64);
                const int rsp = __shfl(rs, from_pos(k - 1), 64);
                if (k < K && p == k && dk) rs = rsp;
            }
            rep = __shfl(idx, from_pos(rs), 64);
            replo = lane_below(rep);
        }
        const bool searching = !done && (p > 0) && !dup;
        const bool tie_lo = replo < rep;  // equal distances go to the lower cluster index
        // |x - vlo| < |x - v|, or <= when the lower cluster wins ties.  One strict comparison serves both: with the
        // two centroids swapped, "<=" is the negation of "<" (a <= b is !(b < a)), so a lane that gives ties to the
        // lower cluster compares the other way round and flips the answer.
        const double c1 = tie_lo ? v : vlo, c2 = tie_lo ? vlo : v;
        auto nearer_raw = [&](float xf) -> bool {
            const double x = (double)xf;
            return fabs(x - c1) < fabs(x - c2);
        };
        auto nearer_lo = [&](float xf) -> bool { return nearer_raw(xf) != tie_lo; };

        // ---- chunk of the boundary: cnt = number of chunks whose first key is nearer to the lower
        // centroid (a prefix of the chunks); invariant lo <= cnt <= hi -----------------------------
        const int rlo = lane_below(r);
        int lo = 0, hi = 0, mode = 0, step = 1;
        if (it == 0) {
            // the starting centroids are the keys at ranks r: the boundary lies in (r_{p-1}, r_p]
            if (searching) {
                lo = (rlo >> 4) + 1;
                hi = (r + 15) >> 4;
            }
        } else {
            // two probes next to the previous answer; a miss gallops away from it
            const int ia = min(max(cold - 1, 0), n1u - 1), ib = min(cold, n1u - 1);
            const bool ta = nearer_lo(w16[ia]), tb = nearer_lo(w16[ib]);
            if (searching) {
                lo = 0;
                hi = n1u;
                bool below = false;
                if (cold >= 1) {
                    if (ta) lo = cold; else { hi = cold - 1; mode = 1; below = true; }
                }
                if (!below && cold < n1u) {
                    if (tb) { lo = cold + 1; mode = 2; } else hi = cold;
                }
            }
        }
        for (;;) {
            const int len = hi - lo;
            if (__ballot(len > 0) == 0) break;
            int mid;
            if (mode == 1) mid = max(lo, hi - step);
            else if (mode == 2) mid = min(hi - 1, lo + step - 1);
            else mid = lo + (len >> 1);
            mid = min(max(mid, 0), n1u - 1);
            const bool t = nearer_lo(w16[mid]);
            if (len > 0) {
                if (t) {
                    lo = mid + 1;
                    if (mode == 2) step <<= 2; else mode = 0;
                } else {
                    hi = mid;
                    if (mode == 1) step <<= 2; else mode = 0;
                }
            }
        }
        if (searching) cold = lo;
        int cl = searching ? lo - 1 : -1;          // chunk that holds the boundary (-1: boundary at rank 0)
        // what the cluster below sees of this position: its chunk, boundary and the sums of the
        // keys of that chunk below the boundary; a position that repeats the value below it owns
        // nothing and passes on what the next distinct position shows
        int xcl = cl;
        if (__builtin_expect(anydup, 0)) {
            if (dup) xcl = (p == K - 1) ? n1u : -2;
            for (int k = 14; k >= 1; --k) {
                const int nx = __shfl(xcl, from_pos(k + 1), 64);
                if (k <= K - 2 && p == k && xcl == -2) xcl = nx;
            }
        }
        int cl_next = lane_above(xcl);
        if (p == K - 1) cl_next = n1u;
        const bool summing = !done && !dup;
        cl_next = max(cl_next, cl);
        // whole chunks between the two boundary chunks: [a0, b0) in chunk units
        int a0 = summing ? cl + 1 : 0, b0 = summing ? cl_next : 0;
        b0 = max(b0, a0);

        // ---- one round of global loads: the boundary chunk's keys and the level-0 pieces ----------
        // (lanes without a boundary chunk read the row's first chunk and ignore it)
        const int rbase = cl * 16;
        const int cl_want = cl >= 0 ? cl : 0;
        const bool reload = cl_want != cl_held;
        if (reload) {
            const u64x2_a8 *kv = (const u64x2_a8 *)(keys + cl_want * 16);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const u64x2 t2 = kv[j];
                el[2 * j] = t2.x;
                el[2 * j + 1] = t2.y;
            }
            cl_held = cl_want;
        }
        const int la0 = min(b0, (a0 + 3) & ~3), rb0 = max(la0, b0 & ~3);
        // (with two wavefronts per SIMD the pieces are requested here, ahead of the work on the keys; with three
        // there are no registers to park them in, and a third wavefront to wait behind)
        double2 pc[6];
        auto load_pieces = [&]() {
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                pc[k] = (a0 + k < la0) ? L1[a0 + k] : make_double2(0.0, 0.0);
                pc[3 + k] = (rb0 + k < b0) ? L1[rb0 + k] : make_double2(0.0, 0.0);
            }
        };
        if (WAVES <= 2) load_pieces();

        int tc = 0;         // (counted with the raw comparison and turned round once for the lanes that flip it)
        if (RAGGED) {
            const int nvalid = m - rbase;   // keys past the end of the row are not this row's
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (j >= nvalid) el[j] = NEUTRAL_KEY;
                tc += (j < nvalid && nearer_raw(elem_w(el[j]))) ? 1 : 0;
            }
            if (tie_lo) tc = min(max(nvalid, 0), 16) - tc;
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) tc += nearer_raw(elem_w(el[j])) ? 1 : 0;
            if (tie_lo) tc = 16 - tc;
        }
        if (cl < 0) tc = 0;
        Bcur = (searching && cl >= 0) ? rbase + tc : 0;  // p == 0 or no chunk below the boundary: 0
        if (__builtin_expect(anydup, 0)) {
            // a position sharing its value with the one before it owns nothing:
            // its range starts where the next distinct value's range starts
            if (dup) Bcur = (p == K - 1) ? m : -1;
            for (int k = 14; k >= 1; --k) {
                const int bn = __shfl(Bcur, from_pos(k + 1), 64);
                if (k <= K - 2 && p == k && Bcur < 0) Bcur = bn;
            }
        }
        {   // the assignment of a bit width is unchanged: every later iteration would repeat this state
            const bool same = (Bcur == Bold) && (idx == idxold);
            const u64 moving = __ballot(!done && !same);
            if (it > 0 && (moving & maskb) == 0) done = true;
        }
        int Bnext = lane_above(done ? Bold : Bcur);
        if (p == K - 1) Bnext = m;
        Bnext = max(Bnext, Bcur);
        if (!done) {
            Bold = Bcur;
            idxold = idx;
        }

        // own chunk: its first tl keys (below the boundary) go to the cluster below, the keys from
        // there up to th (the next boundary, if it falls into this chunk) are this cluster's
        const bool own = searching && cl >= 0;
        const int tl = own ? tc : 0;
        const int th = own ? min(16, Bnext - rbase) : 0;
        double lowD = 0.0, lowN = 0.0, D = 0.0, N = 0.0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float sf = plain_s(el[j]);
            const double wd = (double)elem_w(el[j]);
            // tl <= th: the keys below th minus those below tl are the cluster's own (the difference is s or 0, exactly)
            const float sl = (j < tl) ? sf : 0.0f;
            const float su = (j < th) ? sf : 0.0f;
            const float sh = __fsub_rn(su, sl);
            const double sld = (double)sl, shd = (double)sh;
            lowD += sld;
            lowN = fma(sld, wd, lowN);     // s * w of two floats is exact
            D += shd;
            N = fma(shd, wd, N);
        }
        if (__builtin_expect(anydup, 0)) {
            double xd = lowD, xn = lowN;
            int tag = dup ? ((p == K - 1) ? 1 : -2) : 0;   // -2: waiting for the next distinct position
            if (dup) { xd = 0.0; xn = 0.0; }
            for (int k = 14; k >= 1; --k) {
                const double nd = shfl_d(xd, from_pos(k + 1));
                const double nn = shfl_d(xn, from_pos(k + 1));
                const int nt = __shfl(tag, from_pos(k + 1), 64);
                if (k <= K - 2 && p == k && tag == -2) { xd = nd; xn = nn; tag = nt; }
            }
            lowD = xd;
            lowN = xn;
        }
        if (WAVES > 2) load_pieces();
        double nD = lane_above(lowD), nN = lane_above(lowN);
        if (p == K - 1 || cl_next <= cl) { nD = 0.0; nN = 0.0; }
        D += nD;
        N += nN;
        // level-0 pieces, then the whole groups of 4 chunks in between from the running sums in LDS
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            D += pc[k].x;
            N += pc[k].y;
        }
        {
            int ga = la0 >> 2, gb = rb0 >> 2;
            if (la0 >= rb0) { ga = 0; gb = 0; }
            const double2 da = ppd[ga], db = ppd[gb], na = ppn[ga], nb = ppn[gb];
            D += dd_diff(db, da);
            N += dd_diff(nb, na);
        }
        if (summing) {
            Dk = D;
            Nk = N;
        }
        if (live) emptyk = dup;
        if (summing && !done && D > 0.0) v = quick_div(N, D);
    }

    // ---- row errors from second moments -------------------------------------------------------------
    // sum_j s (w - c)^2 over a cluster = R - 2 c N + c^2 D with R = sum s w^2 over the cluster's final rank
    // range [Bold_p, Bold_{p+1}); D, N are the sums the last iteration formed for the same range.  R comes
    // from the keys of the two partial chunks and the aligned pieces of the second-moment tree.
    double Ep = 0.0, Rp = 0.0;
    {
        const int a = on ? max(Bold, 0) : 0;
        int bnd = lane_above(Bold);
        if (p == K - 1) bnd = m;
        bnd = on ? max(bnd, a) : a;
        const int e0 = min(bnd, (a + 15) & ~15), e1 = max(e0, bnd & ~15);
        const u64x2_a8 *ka = (const u64x2_a8 *)(keys + (a & ~15));        // chunk of a (read whole, masked below)
        const u64x2_a8 *kb = (const u64x2_a8 *)(keys + (e1 < m ? e1 : 0));  // chunk that starts at e1
        u64 ea[16], eb[16];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const u64x2 t2 = ka[j], t3 = kb[j];
            ea[2 * j] = t2.x;
            ea[2 * j + 1] = t2.y;
            eb[2 * j] = t3.x;
            eb[2 * j + 1] = t3.y;
        }
        const int c0 = e0 >> 4, c3 = e1 >> 4;                    // whole chunks [c0, c3)
        const int la0 = min(c3, (c0 + 3) & ~3), rb0 = max(la0, c3 & ~3);
        const double *R1 = prm.R1 + rowc * prm.n1;
        double pr[6];
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            pr[k] = (c0 + k < la0) ? R1[c0 + k] : 0.0;
            pr[3 + k] = (rb0 + k < c3) ? R1[rb0 + k] : 0.0;
        }
        // level 1 (groups of 4 chunks) lives in global memory too: its pieces are requested with the rest
        int ra = la0 >> 2, rb = rb0 >> 2;
        if (la0 >= rb0) { ra = 0; rb = 0; }
        double pq[6];
        {
            const double *RQg = prm.RQ + rowc * prm.nq;
            const int la = min(rb, (ra + 3) & ~3), rbb = max(la, rb & ~3);
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                pq[k] = (ra + k < la) ? RQg[ra + k] : 0.0;
                pq[3 + k] = (rbb + k < rb) ? RQg[rbb + k] : 0.0;
            }
            if (la < rbb) { ra = la >> 2; rb = rbb >> 2; } else { ra = 0; rb = 0; }
        }
        const int abase = a & ~15;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const bool ina = (abase + j >= a) && (abase + j < e0);
            const bool inb = (e1 + j < bnd);
            const double sa = ina ? (double)plain_s(ea[j]) : 0.0, wa = ina ? (double)elem_w(ea[j]) : 0.0;
            const double sb = inb ? (double)plain_s(eb[j]) : 0.0, wb = inb ? (double)elem_w(eb[j]) : 0.0;
            Rp = fma(sa * wa, wa, Rp);
            Rp = fma(sb * wb, wb, Rp);
        }
#pragma unroll
        for (int k = 0; k < 6; ++k) Rp += pr[k];
#pragma unroll
        for (int k = 0; k < 3; ++k) {      // (the order the level loop below adds in: low end, high end, alternating)
            Rp += pq[k];
            Rp += pq[3 + k];
        }
#pragma unroll
        for (int lv = 2; lv < MAX_LEVELS; ++lv) {
            if (lv < LM.nlev && __ballot(ra < rb) != 0) {
                const double *L = (const double *)(blk + LM.roff[lv]);
                const int la = min(rb, (ra + 3) & ~3), rbb = max(la, rb & ~3);
#pragma unroll
                for (int k = 0; k < 3; ++k) {
                    if (ra + k < la) Rp += L[ra + k];
                    if (rbb + k < rb) Rp += L[rbb + k];
                }
                if (la < rbb) { ra = la >> 2; rb = rbb >> 2; } else { ra = 0; rb = 0; }
            }
        }
        if (on && !emptyk && Dk > 0.0) Ep = fma(v, fma(v, Dk, -2.0 * Nk), Rp);
    }
    // per bit width: the clusters' errors added in position order by the lane of position 0
    double *escr = (double *)(smem + 2 * (size_t)LM.bytes);
    __syncthreads();
    escr[lane] = Ep;
    escr[64 + lane] = Rp;
    __syncthreads();
    double err_b = 0.0;
    bool exact_b = false;
    if (on && p == 0) {
        double rtot = 0.0;
        for (int k = 0; k < K; ++k) {
            err_b += escr[lane + k];
            rtot += escr[64 + lane + k];
        }
        // cancellation leaves about 1e-16 * rtot of rounding in err_b: below 1e-9 * rtot (or negative, or
        // not a number) the error is evaluated key by key instead
        exact_b = !(err_b >= 1e-9 * rtot) || !(err_b > 0.0);
    }
    if (on) {
        BitState *o = prm.bstate + row * 4 + (b - 1);
        o->cent[p] = v;
        o->idx[p] = idx;
        o->B[p] = Bold;
        if (p == K - 1) {
            o->B[K] = m;
            o->active = 1;
        }
        if (p == 0) {
            o->err = err_b;
            o->exact = exact_b ? 1 : 0;
        }
    }
    // table mode: centroids, bounds and errors go out from here; finish_kernel only has the flagged errors left
    {
        int b1 = lane_above(Bold);
        if (p == K - 1) b1 = m;
        if (on && !prm.bits) {
            const long long obase = row * prm.stride + ((1 << b) - (1 << prm.bmin));
            const float up = (b1 > Bold) ? elem_w(keys[b1 - 1]) : -INFINITY;
            prm.cent[obase + idx] = v;
            if (prm.upper) prm.upper[obase + idx] = up;
            if (p == 0 && !exact_b) prm.E[row * (prm.bmax - prm.bmin + 1) + (b - prm.bmin)] = err_b;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Kernel 3: errors, centroids, thresholds, labels from the final boundaries.
// ---------------------------------------------------------------------------------------------
constexpr int FIN_THREADS = 256;
constexpr int FIN_WAVES = FIN_THREADS / 64;

__global__ void __launch_bounds__(FIN_THREADS) finish_kernel(ClusterParams prm) {
    __shared__ BitState bs[4];
    __shared__ double red[4 * FIN_WAVES];
    __shared__ float thr[16];
    __shared__ int thl[16];
    const int m = prm.m;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long row = blockIdx.x;
    const u64 *__restrict__ keys = prm.keys + row * (long long)m;
    const int rowbits = prm.bits ? (int)prm.bits[row] : 0;
    if (!prm.bits) {
        // table mode: lloyd_iter_kernel has written everything except the errors it flagged for evaluation key by key
        const BitState *st = prm.bstate + row * 4;
        int todo = 0;
        for (int bi = prm.bmin - 1; bi < prm.bmax; ++bi) todo |= st[bi].exact;
        if (!todo) return;      // (the same for the whole workgroup)
    }
    {
        const int *src = (const int *)(prm.bstate + row * 4);
        int *dst = (int *)bs;
        for (int j = tid; j < (int)(4 * sizeof(BitState) / 4); j += FIN_THREADS) dst[j] = src[j];
    }
    __syncthreads();
    if (tid < 4) {
        const int bb = tid + 1;
        bs[tid].active = prm.bits ? (bb == rowbits) : (bb >= prm.bmin && bb <= prm.bmax);
    }
    __syncthreads();
    // the row errors normally come from the clusters' second moments (lloyd_iter_kernel); a bit width whose
    // error drowned in cancellation there is evaluated key by key below
    int anyexact = 0;
#pragma unroll
    for (int bi = 0; bi < 4; ++bi) anyexact |= __builtin_amdgcn_readfirstlane(bs[bi].active && bs[bi].exact);

    // ---- errors: sum s (w - c)^2 over the sorted row, every key once ----------
    double e4[4] = {0.0, 0.0, 0.0, 0.0};
    // per bit width, the same in every lane: cluster of the first key of the current stretch of 64
    // ranks, the rank where that cluster ends, its centroid
    int pcur[4] = {0, 0, 0, 0}, nxt[4] = {0, 0, 0, 0};
    double ccur[4] = {0.0, 0.0, 0.0, 0.0};
    int act[4];
#pragma unroll
    for (int bi = 0; bi < 4; ++bi) act[bi] = __builtin_amdgcn_readfirstlane(bs[bi].active && bs[bi].exact);
    constexpr int EU = 4;   // stretches of 64 ranks whose loads are in flight together
    for (int base0 = wave * 64; anyexact && base0 < m; base0 += EU * FIN_THREADS) {
        u64 els[EU];
#pragma unroll
        for (int u = 0; u < EU; ++u) {
            const int rk = base0 + u * FIN_THREADS + lane;
            els[u] = (rk < m) ? keys[rk] : NEUTRAL_KEY;   // ranks past the row carry s = 0 and add nothing
        }
#pragma unroll
        for (int u = 0; u < EU; ++u) {
            const int base = base0 + u * FIN_THREADS;
            if (base >= m) break;
            const int rk = base + lane;
            const double w = (double)elem_w(els[u]), s = (double)plain_s(els[u]);
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) {
                if (!act[bi]) continue;
                const int Kb = 2 << bi;
                if (base >= nxt[bi]) {
                    int pp = pcur[bi];
                    while (pp + 1 < Kb && __builtin_amdgcn_readfirstlane(bs[bi].B[pp + 1]) <= base) ++pp;
                    pcur[bi] = pp;
                    nxt[bi] = __builtin_amdgcn_readfirstlane(bs[bi].B[pp + 1]);
                    ccur[bi] = bs[bi].cent[pp];
                }
                double c = ccur[bi];
                if (base + 64 > nxt[bi]) {   // a boundary falls inside this stretch: look the cluster up per lane
                    int pp = pcur[bi];
                    while (pp + 1 < Kb && bs[bi].B[pp + 1] <= rk) ++pp;
                    c = bs[bi].cent[pp];
                }
                const double dlt = w - c;
                e4[bi] += s * dlt * dlt;
            }
        }
    }
#pragma unroll
    for (int bi = 0; bi < 4; ++bi) {
        double x = e4[bi];
        for (int d = 32; d >= 1; d >>= 1) x += __shfl_down(x, d, 64);
        if (lane == 0) red[bi * FIN_WAVES + wave] = x;
    }
    __syncthreads();

    // ---- outputs ------------------------------------------------------------------
    const int nb = prm.bmax - prm.bmin + 1;
    if (wave == 0) {
        for (int bi = 0; bi < 4; ++bi) {
            if (!bs[bi].active) continue;
            const int bb = bi + 1, Kb = 1 << bb;
            double err = bs[bi].err;
            if (bs[bi].exact) {
                err = 0.0;
                for (int w2 = 0; w2 < FIN_WAVES; ++w2) err += red[bi * FIN_WAVES + w2];
            }
            long long obase;
            if (prm.bits) {
                if (lane == 0) prm.E[row] = err;
                obase = row * 16;
            } else {
                if (lane == 0 && bs[bi].exact) prm.E[row * nb + (bb - prm.bmin)] = err;
                continue;       // centroids and bounds were written by lloyd_iter_kernel
            }
            if (lane < Kb) {
                const int k = bs[bi].idx[lane];
                const int b0 = bs[bi].B[lane], b1 = bs[bi].B[lane + 1];
                const float up = (b1 > b0) ? elem_w(keys[b1 - 1]) : -INFINITY;
                prm.cent[obase + k] = bs[bi].cent[lane];
                if (prm.upper) prm.upper[obase + k] = up;
                if (prm.bits) {
                    thr[lane] = up;
                    thl[lane] = k;
                }
            } else if (prm.bits && lane < 16) {
                prm.cent[obase + lane] = 0.0;
                if (prm.upper) prm.upper[obase + lane] = -INFINITY;
                thr[lane] = INFINITY;
                thl[lane] = bs[bi].idx[Kb - 1];
            }
        }
    }
    if (prm.bits && prm.labels) {
        __syncthreads();
        // label of a column: the cluster whose value range holds w~ (ranges are
        // disjoint and ordered by position; empty ones have upper = -inf)
        // thr[0..K) holds the bounds by position; positions are ordered by centroid, and so are the
        // bounds of the non-empty ones.  Empty positions (-inf) are skipped by carrying the running
        // maximum forward, which keeps the array sorted for the binary search.
        if (tid == 0) {
            float run = -INFINITY;
            int lastl = thl[0];
            for (int k = 0; k < 16; ++k) {
                if (thr[k] == -INFINITY) {
                    thr[k] = run;          // an empty range: nothing is <= run that was not caught before
                    thl[k] = lastl;
                } else {
                    run = thr[k];
                    lastl = thl[k];
                }
            }
        }
        __syncthreads();
        const float *Wr = prm.W + row * prm.ld;
        uint8_t *Lr = prm.labels + row * (long long)m;
        for (int j = tid; j < m; j += FIN_THREADS) {
            const float w = Wr[j];
            const float wt = prm.alpha ? __fdiv_rn(w, prm.alpha[j]) : w;
            int pos = (thr[7] < wt) ? 8 : 0;
            pos += (thr[pos + 3] < wt) ? 4 : 0;
            pos += (thr[pos + 1] < wt) ? 2 : 0;
            pos += (thr[pos] < wt) ? 1 : 0;
            Lr[j] = (uint8_t)thl[pos];
        }
    }
}

__global__ void select_kernel(long long n, int bmin, int bmax, const uint8_t *bits, const double *E,
                              const double *cent_all, const float *upper_all, double *cent, float *upper,
                              double *err) {
    const long long i = (long long)blockIdx.x * (blockDim.x / 16) + threadIdx.x / 16;
    const int k = threadIdx.x & 15;
    if (i >= n) return;
    int b = bits[i];
    b = b < bmin ? bmin : (b > bmax ? bmax : b);
    const int nb = bmax - bmin + 1;
    const int stride = (2 << bmax) - (1 << bmin);
    const int off = (1 << b) - (1 << bmin);
    const bool in = k < (1 << b);
    cent[i * 16 + k] = in ? cent_all[i * stride + off + k] : 0.0;
    if (upper) upper[i * 16 + k] = in ? upper_all[i * stride + off + k] : -INFINITY;
    if (err && k == 0) err[i] = E[i * nb + (b - bmin)];
}

// ---------------------------------------------------------------------------------------------
// The least error ANY assignment of a row to at most K clusters can have (K = 2^b): the floor under
// what the Lloyd iterations reach from their quantile start.  In one dimension an optimal assignment
// cuts the sorted values into intervals, so with prefix sums A = sum s, B = sum s w, C = sum s w^2
// over the sorted keys
//     cost(i, j) = (C_j - C_i) - (B_j - B_i)^2 / (A_j - A_i)      (keys i..j-1; 0 without mass)
//     D_1[j] = cost(0, j),   D_k[j] = min_{0 <= i <= j} D_{k-1}[i] + cost(i, j).
// The leftmost minimiser opt_k[j] does not decrease with j (the cost is a Monge array), so every
// layer is filled by halving: j = the odd multiples of a stride h, each searching only
// opt[j - h] .. opt[j + h], for h = 2^(L-1), 2^(L-2), ..., 1.  One workgroup per row walks the
// levels; a level's positions are shared out by the length of their ranges (see OPT_S below).  A, B, C and D live in
// global memory (40 bytes per key: more than the LDS holds), read with consecutive lanes on
// consecutive i; the cuts opt live in LDS when the row is short enough.
// ---------------------------------------------------------------------------------------------
constexpr int OPT_THREADS = 1024;
constexpr int OPT_WAVES = OPT_THREADS / 64;
constexpr int OPT_MAX_WG = 1024;                // workgroups (each with its own scratch) at most

struct OptParams {
    const u64 *keys;     // sorted keys, m per row
    int m, bmin, bmax;
    long long n;
    double *E;           // n x (bmax - bmin + 1)
    double *scratch;     // per workgroup: 5 arrays of mp doubles (A, B, C, D, D') and mp ints (opt)
    long long mp;        // m + 2 rounded up to a multiple of 32
    int opt_in_lds;
};

__device__ __forceinline__ bool opt_less(double a, int ia, double b, int ib) { return a < b || (a == b && ia < ib); }

// min over [lo, hi] of D[i] + cost(i, j) for the candidates of lane r of a team of G lanes (i = lo + r,
// lo + r + G, ...), smallest i among equals.  Four candidates are in flight at once (the loop is bound by the
// latency of its loads); an index past hi is clamped to hi, which only repeats a valid candidate.
__device__ __forceinline__ void opt_scan(const double *__restrict__ A, const double *__restrict__ B,
                                         const double *__restrict__ C, const double *__restrict__ Dp, int j, int lo,
                                         int hi, int r, int G, double &best, int &arg) {
    constexpr int U = 4;
    const double Aj = A[j], Bj = B[j], Cj = C[j];
    best = INFINITY;
    arg = 0x7fffffff;
    for (int i0 = lo + r; i0 <= hi; i0 += U * G) {
        double a[U], b[U], c[U], d[U];
        int idx[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            idx[u] = min(i0 + u * G, hi);
            a[u] = A[idx[u]];
            b[u] = B[idx[u]];
            c[u] = C[idx[u]];
            d[u] = Dp[idx[u]];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const double dA = Aj - a[u], dB = Bj - b[u], dC = Cj - c[u];
            double cost = dA > 0.0 ? dC - quick_div(dB * dB, dA) : 0.0;
            cost = cost > 0.0 ? cost : 0.0;
            const double v = d[u] + cost;
            if (v < best) { best = v; arg = idx[u]; }
        }
    }
}

__device__ __forceinline__ void opt_bounds(const int *opt, int j, int h, int m, int &lo, int &hi) {
    lo = opt[j - h];                          // opt[0] = 0
    hi = (j + h <= m) ? min(opt[j + h], j) : j;
    hi = max(hi, lo);
}

// One position by a team of G lanes (a power of two, at most 64; all lanes of the wave call this together,
// `valid` says whether the team has a position): scan, reduce over the team, lane 0 of the team writes.
__device__ __forceinline__ void opt_team(const double *A, const double *B, const double *C, const double *Dp,
                                         double *Dn, int *opt, int h, int m, bool valid, int q, int r, int G) {
    const int j = valid ? h * (2 * q + 1) : 0;
    double best = INFINITY;
    int arg = 0x7fffffff;
    if (valid) {
        int lo, hi;
        opt_bounds(opt, j, h, m, lo, hi);
        opt_scan(A, B, C, Dp, j, lo, hi, r, G, best, arg);
    }
    for (int o = G >> 1; o >= 1; o >>= 1) {
        const double ob = __shfl_xor(best, o, 64);
        const int oa = __shfl_xor(arg, o, 64);
        if (opt_less(ob, oa, best, arg)) { best = ob; arg = oa; }
    }
    if (valid && r == 0) { Dn[j] = best; opt[j] = arg; }
}

// Ranges of one level differ wildly in length (where the best cut jumps, one position inherits the whole
// jump as its range, on every level), so positions are sorted into four classes by the number of
// candidates: up to OPT_S by one thread, up to OPT_M by 16 lanes, up to OPT_L by a wavefront, longer ones
// by the whole workgroup.
constexpr int OPT_S = 16, OPT_M = 256, OPT_L = 4096;
constexpr int OPT_MCAP = 4096, OPT_LCAP = 256, OPT_XCAP = 16;

__global__ void __launch_bounds__(OPT_THREADS) kmeans_optimal_kernel(OptParams prm) {
    __shared__ double sc[3][OPT_WAVES];
    __shared__ double wb[OPT_XCAP][OPT_WAVES];
    __shared__ int wa[OPT_XCAP][OPT_WAVES];
    __shared__ unsigned short listM[OPT_MCAP], listL[OPT_LCAP], listX[OPT_XCAP];
    __shared__ int cntM[2], cntL[2], cntX[2];
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = prm.m;
    double *A = prm.scratch + (long long)blockIdx.x * (5 * prm.mp + prm.mp / 2);
    double *B = A + prm.mp, *C = B + prm.mp, *D0 = C + prm.mp, *D1 = D0 + prm.mp;
    // the cuts of the current layer: in LDS when the row fits (every level starts by reading two of them)
    int *opt = prm.opt_in_lds ? (int *)smem : (int *)(D1 + prm.mp);
    int L = 1;
    while ((1 << L) < m + 1) ++L;             // positions 1..m < 2^L
    const int chunk = (m + OPT_THREADS - 1) / OPT_THREADS;
    const int Kmax = 1 << prm.bmax;
    const int nb = prm.bmax - prm.bmin + 1;

    if (tid == 0) { cntM[0] = cntM[1] = 0; cntL[0] = cntL[1] = 0; cntX[0] = cntX[1] = 0; }
    int lists = 0;                            // levels done so far, over all layers and rows
    for (long long row = blockIdx.x; row < prm.n; row += gridDim.x) {
        const u64 *keys = prm.keys + row * (long long)m;
        // ---- prefix sums over the sorted keys
        const int j0 = min(m, tid * chunk), j1 = min(m, j0 + chunk);
        double a = 0.0, b = 0.0, c = 0.0;
        for (int j = j0; j < j1; ++j) {
            const u64 el = keys[j];
            const double s = (double)plain_s(el), w = (double)elem_w(el);
            a += s;
            b = fma(s, w, b);
            c = fma(s * w, w, c);
        }
        double ia = a, ib = b, ic = c;        // inclusive scan over the wave, then over the waves
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double ta = __shfl_up(ia, o, 64), tb = __shfl_up(ib, o, 64), tc = __shfl_up(ic, o, 64);
            if (lane >= o) { ia += ta; ib += tb; ic += tc; }
        }
        if (lane == 63) { sc[0][wave] = ia; sc[1][wave] = ib; sc[2][wave] = ic; }
        __syncthreads();
        double pa = ia - a, pb = ib - b, pc = ic - c;     // exclusive within the wave
        for (int w = 0; w < wave; ++w) { pa += sc[0][w]; pb += sc[1][w]; pc += sc[2][w]; }
        if (tid == 0) { A[0] = 0.0; B[0] = 0.0; C[0] = 0.0; D0[0] = 0.0; D1[0] = 0.0; opt[0] = 0; }
        for (int j = j0; j < j1; ++j) {
            const u64 el = keys[j];
            const double s = (double)plain_s(el), w = (double)elem_w(el);
            pa += s;
            pb = fma(s, w, pb);
            pc = fma(s * w, w, pc);
            A[j + 1] = pa; B[j + 1] = pb; C[j + 1] = pc;
            double c1 = pa > 0.0 ? pc - quick_div(pb * pb, pa) : 0.0;
            D0[j + 1] = c1 > 0.0 ? c1 : 0.0;            // one cluster
        }
        __syncthreads();

        double *Dp = D0, *Dn = D1;
        for (int k = 2; k <= Kmax; ++k) {
            for (int lev = 0; lev < L; ++lev) {
                const int h = 1 << (L - 1 - lev);
                const int cnt = (m / h + 1) >> 1;         // odd multiples of h that are <= m
                const int cb = lists & 1;                 // this level's list counters (zeroed a level ago)
                ++lists;
                // short ranges at once, the others onto the lists
                for (int q = tid; q < cnt; q += OPT_THREADS) {
                    const int j = h * (2 * q + 1);
                    int lo, hi;
                    opt_bounds(opt, j, h, m, lo, hi);
                    const int len = hi - lo + 1;
                    int slot = -1;
                    if (len > OPT_L) {
                        slot = atomicAdd(&cntX[cb], 1);
                        if (slot < OPT_XCAP) listX[slot] = (unsigned short)q;
                        else slot = -1;
                    }
                    if (slot < 0 && len > OPT_M) {
                        slot = atomicAdd(&cntL[cb], 1);
                        if (slot < OPT_LCAP) listL[slot] = (unsigned short)q;
                        else slot = -1;
                    }
                    if (slot < 0 && len > OPT_S) {
                        slot = atomicAdd(&cntM[cb], 1);
                        if (slot < OPT_MCAP) listM[slot] = (unsigned short)q;
                        else slot = -1;
                    }
                    if (slot < 0) {                       // short, or a list is full: this thread alone
                        double best;
                        int arg;
                        opt_scan(A, B, C, Dp, j, lo, hi, 0, 1, best, arg);
                        Dn[j] = best;
                        opt[j] = arg;
                    }
                }
                __syncthreads();
                const int nM = min(cntM[cb], OPT_MCAP), nL = min(cntL[cb], OPT_LCAP), nX = min(cntX[cb], OPT_XCAP);
                if (tid == 0) { cntM[cb ^ 1] = 0; cntL[cb ^ 1] = 0; cntX[cb ^ 1] = 0; }
                for (int i0 = 0; i0 < nM; i0 += OPT_THREADS / 16) {
                    const int idx = i0 + (tid >> 4);
                    const bool valid = idx < nM;
                    opt_team(A, B, C, Dp, Dn, opt, h, m, valid, valid ? listM[idx] : 0, tid & 15, 16);
                }
                for (int i0 = 0; i0 < nL; i0 += OPT_WAVES) {
                    const int idx = i0 + wave;
                    const bool valid = idx < nL;
                    opt_team(A, B, C, Dp, Dn, opt, h, m, valid, valid ? listL[idx] : 0, lane, 64);
                }
                if (nX > 0) {
                    for (int x = 0; x < nX; ++x) {
                        const int j = h * (2 * (int)listX[x] + 1);
                        int lo, hi;
                        opt_bounds(opt, j, h, m, lo, hi);
                        double best;
                        int arg;
                        opt_scan(A, B, C, Dp, j, lo, hi, tid, OPT_THREADS, best, arg);
#pragma unroll
                        for (int o = 32; o >= 1; o >>= 1) {
                            const double ob = __shfl_xor(best, o, 64);
                            const int oa = __shfl_xor(arg, o, 64);
                            if (opt_less(ob, oa, best, arg)) { best = ob; arg = oa; }
                        }
                        if (lane == 0) { wb[x][wave] = best; wa[x][wave] = arg; }
                    }
                    __syncthreads();
                    if (tid < nX) {
                        double best = wb[tid][0];
                        int arg = wa[tid][0];
                        for (int w = 1; w < OPT_WAVES; ++w)
                            if (opt_less(wb[tid][w], wa[tid][w], best, arg)) { best = wb[tid][w]; arg = wa[tid][w]; }
                        const int j = h * (2 * (int)listX[tid] + 1);
                        Dn[j] = best;
                        opt[j] = arg;
                    }
                }
                __syncthreads();                           // the level's opt and D are read by the next
            }
            if (tid == 0 && (k & (k - 1)) == 0) {
                int bb = 0;
                while ((1 << bb) < k) ++bb;
                if (bb >= prm.bmin) prm.E[row * nb + (bb - prm.bmin)] = Dn[m];
            }
            double *t = Dp; Dp = Dn; Dn = t;
            __syncthreads();
        }
    }
}

// Input validation (off unless the caller asks for it): bit 0 a non-finite weight, bit 1 a sensitivity that is
// negative or not finite, bit 2 a scale that is not a positive finite number.
__global__ void validate_clear_kernel(int *flag) { *flag = 0; }
__global__ void __launch_bounds__(256) validate_kernel(const float *W, const float *S, const float *alpha, long long n,
                                                      int m, long long ld, int *flag) {
    int bad = 0;
    for (long long row = blockIdx.x; row < n; row += gridDim.x) {
        const float *Wr = W + row * ld, *Sr = S + row * ld;
        for (int j = threadIdx.x; j < m; j += 256) {
            const float w = Wr[j], sv = Sr[j];
            if (!(fabsf(w) < INFINITY)) bad |= 1;
            if (!(sv >= 0.0f && sv < INFINITY)) bad |= 2;
        }
    }
    if (alpha && blockIdx.x == 0) {
        for (int j = threadIdx.x; j < m; j += 256) {
            const float a = alpha[j];
            if (!(a > 0.0f && a < INFINITY)) bad |= 4;
        }
    }
    if (__ballot(bad != 0) && bad) atomicOr(flag, bad);
}

// With validation on: checks W, S and alpha on the device and waits for the answer.
skim_status validate_inputs(skim_ctx *ctx, const ClusterParams &prm, int64_t n) {
    if (!ctx->validate || n == 0) return SKIM_OK;
    hipLaunchKernelGGL(validate_clear_kernel, dim3(1), dim3(1), 0, ctx->stream, prm.vflag);
    long long grid = 8ll * ctx->num_cu;
    if (grid > n) grid = n;
    hipLaunchKernelGGL(validate_kernel, dim3((unsigned)grid), dim3(256), 0, ctx->stream, prm.W, prm.S, prm.alpha,
                       (long long)n, prm.m, prm.ld, prm.vflag);
    SKIM_HIP(ctx, hipGetLastError());
    int flag = 0;
    SKIM_HIP(ctx, hipMemcpyAsync(&flag, prm.vflag, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    SKIM_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (flag)
        SKIM_FAIL(ctx, SKIM_ERR_NONFINITE, "input validation:%s%s%s", (flag & 1) ? " W holds a value that is not finite;" : "",
                  (flag & 2) ? " S holds a value that is negative or not finite;" : "",
                  (flag & 4) ? " alpha holds a value that is not a positive finite number;" : "");
    return SKIM_OK;
}

size_t sort_lds_bytes(int P) { return (size_t)(P + P / 16) * 8; }

size_t lloyd_lds_bytes(int m) { return 2 * (size_t)level_map((m + 15) >> 4).bytes + 128 * sizeof(double); }

// Scratch layout of one call (inside the caller's workspace).
skim_status carve_cluster_ws(skim_ctx *ctx, ClusterParams &prm, int64_t n, double **cent_scratch) {
    prm.nseg = 1;
    prm.seglen = prm.m;
    if (prm.m > SORT_MAX_KEYS) {   // two sorted halves, merged in global memory
        prm.nseg = 2;
        prm.seglen = (((prm.m + 1) / 2) + 15) & ~15;
    }
    int logP = 6;
    while ((1 << logP) < prm.seglen) ++logP;
    if (logP < 10) logP = 10;   // at least 1024 keys = one wavefront of 16-key threads
    prm.logP = logP;
    prm.P = 1 << logP;
    prm.n1 = (prm.nseg == 1) ? prm.P / EPT : (prm.m + 15) / 16;
    skim_ws_cursor cur{(char *)ctx->ws, 0, ctx->ws_bytes};
    prm.keys = (u64 *)cur.take((size_t)n * prm.m * sizeof(u64));
    prm.L1 = (double2 *)cur.take((size_t)n * prm.n1 * sizeof(double2));
    prm.nq = (prm.n1 + 3) / 4;
    prm.Q = (double2 *)cur.take((size_t)n * prm.nq * sizeof(double2));
    prm.R1 = (double *)cur.take((size_t)n * prm.n1 * sizeof(double));
    prm.RQ = (double *)cur.take((size_t)n * prm.nq * sizeof(double));
    prm.w16 = (float *)cur.take((size_t)n * prm.n1 * sizeof(float));
    prm.bstate = (BitState *)cur.take((size_t)n * 4 * sizeof(BitState));
    prm.vflag = (int *)cur.take(256);
    bool ok = prm.keys && prm.L1 && prm.Q && prm.R1 && prm.RQ && prm.w16 && prm.bstate && prm.vflag;
    prm.keys_seg = nullptr;
    prm.segmass = nullptr;
    if (prm.nseg > 1) {
        prm.keys_seg = (u64 *)cur.take((size_t)n * prm.m * sizeof(u64));
        prm.segmass = (int *)cur.take((size_t)n * prm.nseg * sizeof(int));
        ok = ok && prm.keys_seg && prm.segmass;
    }
    if (cent_scratch) {
        *cent_scratch = (double *)cur.take((size_t)n * prm.stride * sizeof(double));
        ok = ok && *cent_scratch;
    }
    if (!ok) SKIM_FAIL(ctx, SKIM_ERR_WORKSPACE, "workspace missing or smaller than skim_workspace_bytes(n, m)");
    return SKIM_OK;
}

// sort_only: stop once the sorted keys (unit weights already put in for rows without mass) are in prm.keys
skim_status launch_cluster(skim_ctx *ctx, ClusterParams &prm, int64_t n, bool sort_only = false) {
    {
        const skim_status vs = validate_inputs(ctx, prm, n);
        if (vs != SKIM_OK) return vs;
    }
    // Threads: one per 8 slots of the padded unit, 1024 at most (and one wavefront at least); fewer key slots per
    // thread leave the compiler more registers.
    int threads = prm.P / 8;
    if (threads > 1024) threads = 1024;
    if (threads < MIN_THREADS) threads = MIN_THREADS;
    // 16-byte loads when every unit starts at a multiple of 16 bytes and has a multiple of 4 columns; then
    // 8, 12 or 16 slots per thread, the least that covers the unit.  Otherwise 4-byte loads and 16 slots.
    const bool vec = ((uintptr_t)prm.W % 16 == 0) && ((uintptr_t)prm.S % 16 == 0) && (prm.ld % 4 == 0) && (prm.m % 4 == 0) &&
                     (prm.seglen % 4 == 0);
    const int per_thread = (prm.seglen + threads - 1) / threads;
    const int variant = !vec ? 3 : (per_thread <= 8 ? 0 : (per_thread <= 12 ? 1 : 2));
    // (what the kernel variants rely on for the networks compiled into them)
    if ((variant == 0 && prm.logP > 13) || ((variant == 1 || variant == 2) && prm.logP != 14))
        SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "internal: sort variant %d does not serve a padded length of 2^%d", variant, prm.logP);
    size_t lds = sort_lds_bytes(prm.P);
    if ((int64_t)lds > ctx->lds_limit)
        SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "row length %d needs %zu bytes of LDS, device allows %d", prm.m, lds, ctx->lds_limit);
    // bucket path: the keys of one unit (seglen at most), two bytes per value bin, the coarse tables.
    // About 1.4 bins per key or more (at most 32768 bins: a bin index takes 15 bits): with fewer, too many rows
    // would find a bin of more than BIN_MAX_KEYS keys and sort twice; with many more, clearing and scanning the
    // counters costs more than the rare second sort.
    prm.bk_bpt = 0;
    {
        const size_t key_bytes = (((size_t)prm.seglen + prm.seglen / 16 + 1) * 8 + 15) & ~(size_t)15;
        const size_t base_lds = lds;
        int best_per_cu = 0;
        for (int bpt = 8; bpt <= 32; bpt += 8) {
            // a thread's block of counters is bpt / 2 words; blocks of 8, 16 or 32 words get 4 spare words each,
            // so that 8 neighbouring threads' 16-byte accesses fall into different banks (24 words do already)
            const int pad = (bpt == 24) ? 0 : 4;
            const size_t hist_bytes = (size_t)(bpt / 2 + pad) * threads * 4;
            const size_t need = key_bytes + hist_bytes + BK_COARSE_BYTES + BK_MISC_BYTES;
            const long long bins = (long long)bpt * threads - COARSE_N - 16;
            if (need + 1024 > (size_t)ctx->lds_limit || 10ll * prm.seglen > 7ll * bins || bpt * threads > 32768) continue;
            // workgroups a compute unit holds with this choice (threads and LDS); more of them beats more bins
            const size_t total = need > base_lds ? need : base_lds;
            int per_cu = (int)((size_t)ctx->lds_limit / (total + 256));
            if (per_cu > 2048 / threads) per_cu = 2048 / threads;
            if (per_cu <= best_per_cu) continue;
            best_per_cu = per_cu;
            prm.bk_bpt = bpt;
            prm.bk_pad = pad;
            prm.bk_lgbpt = bpt == 8 ? 3 : (bpt == 16 ? 4 : 5);
            prm.bk_hist_off = (uint32_t)key_bytes;
            prm.bk_coarse_off = (uint32_t)(key_bytes + hist_bytes);
            prm.bk_misc_off = prm.bk_coarse_off + BK_COARSE_BYTES;
            lds = total;
        }
    }
    const void *kern = variant == 0 ? (const void *)sort_kernel<8, true>
                     : variant == 1 ? (const void *)sort_kernel<12, true>
                     : variant == 2 ? (const void *)sort_kernel<16, true> : (const void *)sort_kernel<16, false>;
    if (lds > 65536 && lds > ctx->sort_lds_enabled[variant]) {
        SKIM_HIP(ctx, hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        ctx->sort_lds_enabled[variant] = lds;
    }
    if (n == 0) return SKIM_OK;
    if ((int64_t)n * prm.nseg > 0x7fffffff) SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "too many rows");
    prm.nwork = (long long)n * prm.nseg;
    prm.work_counters = ctx->sort_counters;
    // as many workgroups as the device holds at once (LDS and thread limits), each looping over its units
    int per_cu = (int)(ctx->lds_limit / (int64_t)(lds + 256));   // (+ the kernel's small static LDS)
    if (per_cu > 2048 / threads) per_cu = 2048 / threads;
    if (per_cu < 1) per_cu = 1;
    if (per_cu > 8) per_cu = 8;
    long long sort_grid = (long long)ctx->num_cu * per_cu;
    if (sort_grid > prm.nwork) sort_grid = prm.nwork;
    if (ctx->profiling) SKIM_HIP(ctx, hipEventRecord(ctx->ev[0], ctx->stream));
    if (variant == 0) hipLaunchKernelGGL((sort_kernel<8, true>), dim3((unsigned)sort_grid), dim3(threads), lds, ctx->stream, prm);
    else if (variant == 1) hipLaunchKernelGGL((sort_kernel<12, true>), dim3((unsigned)sort_grid), dim3(threads), lds, ctx->stream, prm);
    else if (variant == 2) hipLaunchKernelGGL((sort_kernel<16, true>), dim3((unsigned)sort_grid), dim3(threads), lds, ctx->stream, prm);
    else hipLaunchKernelGGL((sort_kernel<16, false>), dim3((unsigned)sort_grid), dim3(threads), lds, ctx->stream, prm);
    if (prm.nseg > 1) {
        const int tiles = (prm.m + MG_TILE - 1) / MG_TILE;
        if ((int64_t)n * tiles > 0x7fffffff) SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "too many rows");
        hipLaunchKernelGGL(merge_tile_kernel, dim3((unsigned)(n * tiles)), dim3(MG_THREADS), 0, ctx->stream, prm, tiles);
    }
    if (sort_only) {
        SKIM_HIP(ctx, hipGetLastError());
        return SKIM_OK;
    }
    if (ctx->profiling) SKIM_HIP(ctx, hipEventRecord(ctx->ev[1], ctx->stream));
    const LevelMap lm = level_map((prm.m + 15) >> 4);
    {
        // Two wavefronts per SIMD = up to 8 workgroups per compute unit, three = up to 12, both as far as the LDS
        // has room.  A workgroup's time hardly depends on how many are resident, so the kernel takes as many rounds of
        // workgroups as it needs to seat them all; the three-wavefront variant (about an eighth slower per round)
        // is taken when it saves more rounds than that.
        const size_t llds = lloyd_lds_bytes(prm.m);
        const long long wgs = (n + 1) / 2;
        const long long fit = (long long)((size_t)ctx->lds_limit / (llds + 256));
        const long long seats2 = ctx->num_cu * max(1ll, min(8ll, fit)), seats3 = ctx->num_cu * max(1ll, min(12ll, fit));
        const long long rounds2 = (wgs + seats2 - 1) / seats2, rounds3 = (wgs + seats3 - 1) / seats3;
        const bool three = 9 * rounds3 < 8 * rounds2;
        const dim3 grid((unsigned)wgs), block(ITER_THREADS);
        if (prm.m & 15) {
            if (three) hipLaunchKernelGGL((lloyd_iter_kernel<true, 3>), grid, block, llds, ctx->stream, prm, (long long)n, lm);
            else hipLaunchKernelGGL((lloyd_iter_kernel<true, 2>), grid, block, llds, ctx->stream, prm, (long long)n, lm);
        } else {
            if (three) hipLaunchKernelGGL((lloyd_iter_kernel<false, 3>), grid, block, llds, ctx->stream, prm, (long long)n, lm);
            else hipLaunchKernelGGL((lloyd_iter_kernel<false, 2>), grid, block, llds, ctx->stream, prm, (long long)n, lm);
        }
    }
    hipLaunchKernelGGL(finish_kernel, dim3((unsigned)n), dim3(FIN_THREADS), 0, ctx->stream, prm);
    if (ctx->profiling) {
        SKIM_HIP(ctx, hipEventRecord(ctx->ev[2], ctx->stream));
        ctx->ev_valid = 1;
    }
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}

}  // namespace

extern "C" skim_status skim_error_table(skim_ctx *ctx, const float *W, const float *S, const float *alpha,
                                        int64_t n, int64_t m, int64_t ld, int bmin, int bmax, int iters,
                                        double *E, double *centroids_all, float *upper_all) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!W || !S || !E) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_error_table: W, S and E must not be NULL");
    if (bmin < 1 || bmax > SKIM_MAX_BITS || bmin > bmax) SKIM_FAIL(ctx, SKIM_ERR_ARG, "bit range [%d,%d] outside 1..4", bmin, bmax);
    if (iters < 1) SKIM_FAIL(ctx, SKIM_ERR_ARG, "iters must be >= 1");
    if (n < 0 || n > 0x7fffffff) SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "n = %lld out of range", (long long)n);
    if (m < (1 << bmax) || m > SKIM_MAX_M || ld < m)
        SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "need 2^bmax <= m <= %d and ld >= m (m=%lld, ld=%lld)", SKIM_MAX_M, (long long)m, (long long)ld);
    ClusterParams prm{};
    prm.W = W; prm.S = S; prm.alpha = alpha; prm.ld = ld; prm.m = (int)m; prm.iters = iters;
    prm.bmin = bmin; prm.bmax = bmax; prm.bits = nullptr; prm.E = E;
    prm.stride = (2 << bmax) - (1 << bmin);
    // the kernel always records centroids; give it a place when the caller wants none
    double *scratch = nullptr;
    if ((st = carve_cluster_ws(ctx, prm, n, centroids_all ? nullptr : &scratch)) != SKIM_OK) return st;
    prm.cent = centroids_all ? centroids_all : scratch;
    prm.upper = upper_all;
    prm.labels = nullptr;
    return launch_cluster(ctx, prm, n);
}

extern "C" skim_status skim_cluster_rows(skim_ctx *ctx, const float *W, const float *S, const float *alpha,
                                         int64_t n, int64_t m, int64_t ld, const uint8_t *bits, int iters,
                                         uint8_t *labels, double *centroids, float *upper, double *err) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!W || !S || !bits || !centroids || !err) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_cluster_rows: W, S, bits, centroids, err must not be NULL");
    if (iters < 1) SKIM_FAIL(ctx, SKIM_ERR_ARG, "iters must be >= 1");
    if (n < 0 || n > 0x7fffffff) SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "n = %lld out of range", (long long)n);
    if (m < SKIM_MAX_K || m > SKIM_MAX_M || ld < m)
        SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "need 16 <= m <= %d and ld >= m (m=%lld, ld=%lld)", SKIM_MAX_M, (long long)m, (long long)ld);
    ClusterParams prm{};
    prm.W = W; prm.S = S; prm.alpha = alpha; prm.ld = ld; prm.m = (int)m; prm.iters = iters;
    prm.bmin = 1; prm.bmax = 4; prm.bits = bits; prm.E = err; prm.cent = centroids; prm.upper = upper;
    prm.labels = labels; prm.stride = 16;
    if ((st = carve_cluster_ws(ctx, prm, n, nullptr)) != SKIM_OK) return st;
    return launch_cluster(ctx, prm, n);
}

extern "C" size_t skim_kmeans_optimal_scratch_bytes(int64_t n, int64_t m) {
    if (n < 1 || m < 1 || m > SKIM_MAX_M) return 0;
    const size_t mp = ((size_t)m + 2 + 31) & ~(size_t)31;
    const size_t wgs = n < OPT_MAX_WG ? (size_t)n : (size_t)OPT_MAX_WG;
    return wgs * mp * 44 + 256;
}

extern "C" skim_status skim_kmeans_optimal(skim_ctx *ctx, const float *W, const float *S, const float *alpha,
                                           int64_t n, int64_t m, int64_t ld, int bmin, int bmax, double *E_opt,
                                           void *scratch, size_t scratch_bytes) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!W || !S || !E_opt || !scratch) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_kmeans_optimal: NULL argument");
    if (bmin < 1 || bmax > SKIM_MAX_BITS || bmin > bmax) SKIM_FAIL(ctx, SKIM_ERR_ARG, "bit range [%d,%d] outside 1..4", bmin, bmax);
    if (n < 1 || n > 0x7fffffff) SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "n = %lld out of range", (long long)n);
    if (m < (1 << bmax) || m > SKIM_MAX_M || ld < m)
        SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "need 2^bmax <= m <= %d and ld >= m (m=%lld, ld=%lld)", SKIM_MAX_M, (long long)m, (long long)ld);
    if (((uintptr_t)scratch & 255) != 0) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_kmeans_optimal: scratch not 256-byte aligned");
    const size_t need = skim_kmeans_optimal_scratch_bytes(n, m);
    if (scratch_bytes < need)
        SKIM_FAIL(ctx, SKIM_ERR_WORKSPACE, "skim_kmeans_optimal: scratch of %zu bytes, %zu needed", scratch_bytes, need);
    ClusterParams prm{};
    prm.W = W; prm.S = S; prm.alpha = alpha; prm.ld = ld; prm.m = (int)m; prm.iters = 1;
    prm.bmin = bmin; prm.bmax = bmax; prm.stride = (2 << bmax) - (1 << bmin);
    if ((st = carve_cluster_ws(ctx, prm, n, nullptr)) != SKIM_OK) return st;
    if ((st = launch_cluster(ctx, prm, n, true)) != SKIM_OK) return st;
    OptParams op{};
    op.keys = prm.keys; op.m = (int)m; op.bmin = bmin; op.bmax = bmax; op.n = n; op.E = E_opt;
    op.scratch = (double *)scratch;
    op.mp = ((long long)m + 2 + 31) & ~31ll;
    long long grid = 2ll * ctx->num_cu;
    if (grid > OPT_MAX_WG) grid = OPT_MAX_WG;
    if (grid > n) grid = n;
    const size_t opt_lds = (size_t)op.mp * sizeof(int);
    op.opt_in_lds = opt_lds <= 65536 - 16384;     // no more than the default limit, with the static arrays
    hipLaunchKernelGGL(kmeans_optimal_kernel, dim3((unsigned)grid), dim3(OPT_THREADS), op.opt_in_lds ? opt_lds : 0,
                       ctx->stream, op);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}

extern "C" skim_status skim_select_allocated(skim_ctx *ctx, int64_t n, int bmin, int bmax, const uint8_t *bits,
                                             const double *E, const double *centroids_all, const float *upper_all,
                                             double *centroids, float *upper, double *err) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!bits || !centroids_all || !centroids) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_select_allocated: NULL argument");
    if ((upper && !upper_all) || (err && !E)) SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_select_allocated: output requested without its source");
    if (bmin < 1 || bmax > SKIM_MAX_BITS || bmin > bmax) SKIM_FAIL(ctx, SKIM_ERR_ARG, "bit range [%d,%d] outside 1..4", bmin, bmax);
    if (n <= 0) return SKIM_OK;
    const int rows_per_block = 16;
    hipLaunchKernelGGL(select_kernel, dim3((unsigned)((n + rows_per_block - 1) / rows_per_block)), dim3(256), 0,
                       ctx->stream, (long long)n, bmin, bmax, bits, E, centroids_all, upper_all, centroids, upper, err);
    SKIM_HIP(ctx, hipGetLastError());
    return SKIM_OK;
}
