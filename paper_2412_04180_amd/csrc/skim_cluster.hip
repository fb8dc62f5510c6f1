// Per-row sensitivity-weighted 1-D K-means (Alg. 3 lines 2-10 and 12-15; the
// re-clustering of W * alpha^-1 in Alg. 2) for gfx950.
//
// One workgroup owns one row.  The row's (w~, s~) pairs are staged in LDS as
// 64-bit keys (order-preserving image of w~ in the high word, bits of s~ in the
// low word), sorted once, and float64 sums of s~ and s~ w~ are kept per aligned
// 16-element chunk and 256-element block of the sorted order.  In sorted order
// every cluster of a 1-D K-means is a contiguous rank range, so one Lloyd
// iteration is: per pair of neighbouring centroids a search for the rank where
// the nearer centroid changes, then centroid = (sum of s~ w~) / (sum of s~) over
// the range, assembled from those aligned pieces.  The four bit widths run
// concurrently, one wavefront each, on the same sorted row.
//
// Arithmetic on every decision path is float64 and uses the same predicates as
// the definition: |w - c_lo| versus |w - c_hi| with the lower cluster index
// winning equal distances; centroids with no weight mass keep their value.
#include "skim_common.h"

#include <math.h>

typedef unsigned long long u64;

namespace {

constexpr int EPT = 16;           // sorted elements owned by one thread
constexpr int MIN_THREADS = 256;
constexpr unsigned long long NEUTRAL_KEY = 0x8000000000000000ull;  // encodes (w = +0, s = +0)  // four wavefronts: one per bit width in the Lloyd phase

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
};

struct BitState {  // what the Lloyd wavefront of one bit width leaves for the epilogue
    double cent[16];  // by sorted position
    int idx[16];      // cluster index at that position
    int B[17];        // first rank of each position's range, B[K] = m
    int active;
};

__device__ __forceinline__ uint32_t swz(uint32_t i) { return i ^ ((i >> 4) & 15u); }

__device__ __forceinline__ uint32_t w_to_key(float w) {
    if (w == 0.0f) w = 0.0f;  // -0 and +0 are one value
    uint32_t u = __float_as_uint(w);
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float key_to_w(uint32_t k) {
    uint32_t u = k ^ ((k >> 31) ? 0x80000000u : 0xFFFFFFFFu);
    return __uint_as_float(u);
}
__device__ __forceinline__ float elem_w(u64 e) { return key_to_w((uint32_t)(e >> 32)); }
__device__ __forceinline__ float elem_s(u64 e) { return __uint_as_float((uint32_t)e); }

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

__device__ __forceinline__ void ce(u64 &a, u64 &b, bool desc) {
    const bool sw = (a > b) != desc;
    const u64 x = sw ? b : a;
    const u64 y = sw ? a : b;
    a = x;
    b = y;
}

// One pass over LDS of the bitonic network: the thread holds the 16 elements
// whose indices differ in bits [wb, wb+4) and runs the compare-exchange stages
// of merge size 2^klog for index bits wb+RB_HI down to wb+RB_LO.
template <int RB_HI, int RB_LO>
__device__ __forceinline__ void sort_round(u64 *lds, uint32_t t, int wb, int klog) {
    const uint32_t lowmask = (1u << wb) - 1u;
    const uint32_t base = ((t >> wb) << (wb + 4)) | (t & lowmask);
    u64 v[EPT];
#pragma unroll
    for (int r = 0; r < EPT; ++r) v[r] = lds[swz(base | ((uint32_t)r << wb))];
#pragma unroll
    for (int rb = RB_HI; rb >= RB_LO; --rb) {
#pragma unroll
        for (int r = 0; r < EPT; ++r) {
            if (!(r & (1 << rb))) {
                const uint32_t i = base | ((uint32_t)r << wb);
                const bool desc = (i >> klog) & 1u;
                ce(v[r], v[r | (1 << rb)], desc);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < EPT; ++r) lds[swz(base | ((uint32_t)r << wb))] = v[r];
}

// The merges of size 2, 4, 8, 16 in one pass (index bits 0..3 are in-thread).
__device__ __forceinline__ void sort_first_round(u64 *lds, uint32_t t) {
    const uint32_t base = t << 4;
    u64 v[EPT];
#pragma unroll
    for (int r = 0; r < EPT; ++r) v[r] = lds[swz(base | (uint32_t)r)];
#pragma unroll
    for (int klog = 1; klog <= 4; ++klog) {
#pragma unroll
        for (int rb = klog - 1; rb >= 0; --rb) {
#pragma unroll
            for (int r = 0; r < EPT; ++r) {
                if (!(r & (1 << rb))) {
                    const uint32_t i = base | (uint32_t)r;
                    const bool desc = (i >> klog) & 1u;
                    ce(v[r], v[r | (1 << rb)], desc);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < EPT; ++r) lds[swz(base | (uint32_t)r)] = v[r];
}

__device__ __forceinline__ void dispatch_round(u64 *lds, uint32_t t, int wb, int rb_hi, int rb_lo, int klog) {
    switch (rb_hi * 4 + rb_lo) {
        case 0: sort_round<0, 0>(lds, t, wb, klog); break;
        case 4: sort_round<1, 0>(lds, t, wb, klog); break;
        case 5: sort_round<1, 1>(lds, t, wb, klog); break;
        case 8: sort_round<2, 0>(lds, t, wb, klog); break;
        case 9: sort_round<2, 1>(lds, t, wb, klog); break;
        case 10: sort_round<2, 2>(lds, t, wb, klog); break;
        case 12: sort_round<3, 0>(lds, t, wb, klog); break;
        case 13: sort_round<3, 1>(lds, t, wb, klog); break;
        case 14: sort_round<3, 2>(lds, t, wb, klog); break;
        case 15: sort_round<3, 3>(lds, t, wb, klog); break;
        default: break;
    }
}

// Bitonic sort of P = 2^logP keys in LDS, P/16 working threads.
__device__ void sort_row(u64 *lds, int logP, uint32_t tid) {
    const uint32_t nwork = 1u << (logP - 4);
    const int topbase = (logP >> 2) << 2;  // bits >= topbase live in the shifted top window when logP % 4 != 0
    if (tid < nwork) sort_first_round(lds, tid);
    __syncthreads();
    for (int klog = 5; klog <= logP; ++klog) {
        int b = klog - 1;
        while (b >= 0) {
            int wb, lo;
            if ((logP & 3) && b >= topbase) {
                wb = logP - 4;
                lo = topbase;
            } else {
                wb = (b >> 2) << 2;
                lo = wb;
            }
            if (tid < nwork) dispatch_round(lds, tid, wb, b - wb, lo - wb, klog);
            __syncthreads();
            b = lo - 1;
        }
    }
}

__device__ __forceinline__ double shfl_d(double x, int src) { return __shfl(x, src, 64); }

// Cross-lane moves that stay inside the VALU (DPP): lane i reads lane i^1, lane i^2, its
// mirror inside its group of 8, its mirror inside its row of 16.
template <int CTRL>
__device__ __forceinline__ double dpp_move_d(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

// Sum over the G consecutive lanes of a group; every lane of the group gets the same bits
// (each step adds a lane's value and its partner's, and the partner adds the same two).
template <int G>
__device__ __forceinline__ double group_sum(double x) {
    if (G >= 2) x += dpp_move_d<0xB1>(x);    // quad_perm [1,0,3,2]
    if (G >= 4) x += dpp_move_d<0x4E>(x);    // quad_perm [2,3,0,1]
    if (G >= 8) x += dpp_move_d<0x141>(x);   // row_half_mirror
    if (G >= 16) x += dpp_move_d<0x140>(x);  // row_mirror
    if (G >= 32) x += __shfl_xor(x, 16, 64);
    return x;
}

// Sums of s and s*w over the sorted ranks [a, b), shared out over the G lanes of
// a group (lane g) and reduced so that every lane of the group gets the result.
// The range is cut into aligned pieces whose sums were each formed from their
// own members only (single elements, 16-element chunks, 256-element blocks):
// nothing outside [a, b) enters, so a cluster of tiny weight mass next to a
// heavy element keeps full relative precision (a difference of running prefix
// sums would not).
template <int G>
__device__ __forceinline__ void range_sum(const u64 *sorted, const double2 *csum, const double2 *bsum, int a,
                                          int b, int g, double &D, double &N) {
    constexpr int T = (16 + G - 1) / G;   // loads per lane that cover one 16-wide piece
    // piece boundaries: elements [a, e0) and [e1, b); chunks [c0, c1) and [c2, c3); blocks [b0, b1)
    const int e0 = min(b, (a + 15) & ~15);
    const int e1 = max(e0, b & ~15);
    const int c0 = e0 >> 4, c3 = e1 >> 4;
    const int c1 = (c0 < c3) ? min(c3, (c0 + 15) & ~15) : c0;
    const int c2 = (c0 < c3) ? max(c1, c3 & ~15) : c0;
    const int b0 = c1 >> 4, b1 = (c0 < c3) ? (c2 >> 4) : b0;
    // issue every load first (predicated), then add in a fixed order: one LDS round trip
    u64 el[2 * T];
    double2 ch[2 * T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int r0 = a + g + t * G, r1 = e1 + g + t * G;
        el[t] = (r0 < e0) ? sorted[swz((uint32_t)r0)] : NEUTRAL_KEY;
        el[T + t] = (r1 < b) ? sorted[swz((uint32_t)r1)] : NEUTRAL_KEY;
        const int q0 = c0 + g + t * G, q1 = c2 + g + t * G;
        ch[t] = (q0 < c1) ? csum[q0] : make_double2(0.0, 0.0);
        ch[T + t] = (q1 < c3 && c0 < c3) ? csum[q1] : make_double2(0.0, 0.0);
    }
    double d = 0.0, n = 0.0;
#pragma unroll
    for (int t = 0; t < 2 * T; ++t) {
        // a skipped slot holds (w = +0, s = +0) and adds nothing
        const double s = (double)elem_s(el[t]);
        d += s;
        n = fma(s, (double)elem_w(el[t]), n);
    }
#pragma unroll
    for (int t = 0; t < 2 * T; ++t) {
        d += ch[t].x;
        n += ch[t].y;
    }
    for (int q = b0 + g; q < b1; q += G) {   // whole 256-element blocks (only for ranges beyond 4096 ranks)
        const double2 t = bsum[q];
        d += t.x;
        n += t.y;
    }
    D = group_sum<G>(d);
    N = group_sum<G>(n);
}

// First rank whose inclusive running sum of s reaches tau (weighted-quantile start).
// cpre[q] = running sum of s over the ranks before chunk q.
__device__ __forceinline__ int quantile_rank(const u64 *sorted, const double *cpre, int m, double tau) {
    const int nchunk = (m + 15) >> 4;
    int lo = 0, hi = nchunk - 1;  // largest q with cpre[q] < tau; cpre[0] = 0 < tau
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (cpre[mid] < tau) lo = mid; else hi = mid - 1;
    }
    double acc = cpre[lo];
    const int r0 = lo * 16;
    int found = min(r0 + 15, m - 1);
    for (int j = 0; j < 16; ++j) {
        const int r = r0 + j;
        if (r >= m) break;
        acc += (double)elem_s(sorted[swz((uint32_t)r)]);
        if (acc >= tau) {
            found = r;
            break;
        }
    }
    return found;
}

// Lloyd iterations for one bit width (K = 2^B centroids) on one wavefront.  Position p
// (sorted order of centroid values) is handled by the G = 64/K lanes [p*G, (p+1)*G), which
// search its lower boundary together: first a round of probes around the boundary of the
// previous iteration, then a (G+1)-ary search of what is left.
template <int B>
__device__ void lloyd_wave(const u64 *sorted, const double2 *csum, const double2 *bsum, const double *cpre, int m,
                           int iters, double total, BitState *out) {
    constexpr int K = 1 << B, GS = 6 - B, G = 1 << GS, HALF = G / 2, HM1 = (HALF > 1) ? HALF - 1 : 1;
    constexpr u64 gmask = (1ull << G) - 1ull;
    const int lane = threadIdx.x & 63;
    const int p = lane >> GS;
    const int g = lane & (G - 1);

    // weighted-quantile start with strictly increasing ranks
    const double tau = total * (double)(2 * p + 1) / (double)(2 * K);
    int r = quantile_rank(sorted, cpre, m, tau);
    int prev = -1;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        int rk = __builtin_amdgcn_readlane(r, k << GS);
        rk = max(rk, prev + 1);
        rk = min(rk, m - K + k);
        if (p == k) r = rk;
        prev = rk;
    }
    double v = (double)elem_w(sorted[swz((uint32_t)r)]);
    int idx = p;
    int Bcur = 0, Bold = -1, idxold = -1, Wd = 2;

    // offset of probe gg of the warm round relative to the previous boundary:
    // HALF probes in [-Wd, -1], HALF probes in [0, Wd-1], ascending in gg
    auto warm_off = [&](int gg) -> int {
        return gg < HALF ? -1 - ((HALF - 1 - gg) * (Wd - 1)) / HM1 : ((gg - HALF) * (Wd - 1)) / HM1;
    };

    for (int it = 0; it < iters; ++it) {
        double vlo = shfl_d(v, lane - G);
        int ilo = __shfl(idx, lane - G, 64);
        {   // keep positions ordered by (value, cluster index)
            const bool ok = (p == 0) || (vlo < v) || (vlo == v && ilo < idx);
            if (__ballot(!ok)) {
                int rank = 0;
                for (int q = 0; q < K; ++q) {
                    const double vq = shfl_d(v, q << GS);
                    const int iq = __shfl(idx, q << GS, 64);
                    rank += (vq < v || (vq == v && iq < idx)) ? 1 : 0;
                }
                int src = 0;
                for (int q = 0; q < K; ++q) {
                    const int rq = __shfl(rank, q << GS, 64);
                    if (rq == p) src = q;
                }
                v = shfl_d(v, src << GS);
                idx = __shfl(idx, src << GS, 64);
                vlo = shfl_d(v, lane - G);
                ilo = __shfl(idx, lane - G, 64);
            }
        }
        const bool dup = (p > 0) && (vlo == v);
        int rep = idx;       // lowest cluster index among the positions sharing this value
        const bool anydup = __ballot(dup) != 0;
        int replo = ilo;
        if (anydup) {
            int rs = p;      // first position of this position's run of equal values
            for (int k = 1; k < K; ++k) {
                const int d = __shfl((int)dup, k << GS, 64);
                const int rsp = __shfl(rs, (k - 1) << GS, 64);
                if (p == k && d) rs = rsp;
            }
            rep = __shfl(idx, rs << GS, 64);
            replo = __shfl(rep, lane - G, 64);
        }
        const bool searching = (p > 0) && !dup;
        const bool tie_lo = replo < rep;  // equal distances go to the lower cluster index
        auto nearer_lo = [&](int rank) -> bool {
            const double x = (double)elem_w(sorted[swz((uint32_t)rank)]);
            const double dl = fabs(x - vlo), dh = fabs(x - v);
            return tie_lo ? (dl <= dh) : (dl < dh);
        };

        // first rank that is not nearer to the lower centroid: invariant lo <= answer <= hi
        int lo = 0, hi = searching ? m : 0;
        if (it > 0) {
            const int pr = min(max(Bold + warm_off(g), 0), m - 1);
            const bool pt = searching && nearer_lo(pr);
            const u64 bal = __ballot(pt);
            const int tc = __popcll((bal >> (p << GS)) & gmask);
            if (searching) {
                if (tc > 0) lo = min(max(Bold + warm_off(tc - 1), 0), m - 1) + 1;
                if (tc < G) hi = min(max(Bold + warm_off(tc), 0), m - 1);
            }
        }
        for (;;) {
            const int len = hi - lo;
            if (__ballot(len > 0) == 0) break;
            const int pr = lo + ((g + 1) * len) / (G + 1);
            const bool pt = (len > 0) && nearer_lo(pr);
            const u64 bal = __ballot(pt);
            const int tc = __popcll((bal >> (p << GS)) & gmask);
            const int pl = lo + (tc * len) / (G + 1);
            const int ph = lo + ((tc + 1) * len) / (G + 1);
            if (len > 0) {
                if (tc > 0) lo = pl + 1;
                if (tc < G) hi = ph;
            }
        }
        Bcur = lo;  // p == 0: 0
        if (anydup) {
            // a position sharing its value with the one before it owns nothing:
            // its range starts where the next distinct value's range starts
            if (dup) Bcur = (p == K - 1) ? m : -1;
            for (int k = K - 2; k >= 1; --k) {
                const int bn = __shfl(Bcur, (k + 1) << GS, 64);
                if (p == k && Bcur < 0) Bcur = bn;
            }
        }
        // the assignment is unchanged: every later iteration would repeat this state
        const bool same = (Bcur == Bold) && (idx == idxold);
        if (it > 0 && __ballot(!same) == 0) break;
        {   // next warm round: twice the last move, at least 2
            const int mv = (Bold < 0) ? (m >> B) : abs(Bcur - Bold);
            Wd = min(max(2 * mv + 2, 2), 1 << 14);
        }
        Bold = Bcur;
        idxold = idx;

        // (the shuffle must run with every lane active: no lane-dependent branch around it)
        int Bnext = __shfl(Bcur, lane + G, 64);
        if (p == K - 1) Bnext = m;
        double D, N;
        range_sum<G>(sorted, csum, bsum, Bcur, Bnext, g, D, N);
        if (D > 0.0) v = N / D;
    }

    if (g == 0) {
        out->cent[p] = v;
        out->idx[p] = idx;
        out->B[p] = Bold;
        if (p == K - 1) out->B[K] = m;
    }
}

__global__ void __launch_bounds__(1024) cluster_kernel(ClusterParams prm) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int P = prm.P, m = prm.m;
    const int nchunkP = P >> 4;
    u64 *sorted = (u64 *)smem;
    double2 *csum = (double2 *)(smem + (size_t)P * 8);               // per 16-element chunk: (sum s, sum s*w)
    double2 *bsum = csum + nchunkP;                                  // per 256-element block (at least one entry)
    double *cpre = (double *)(bsum + ((nchunkP + 15) >> 4));         // nchunkP + 1 running sums of s
    double *wtot = cpre + nchunkP + 1;                               // 16 wave totals + 1
    BitState *bs = (BitState *)(wtot + 17);                          // 4 entries
    double *red = (double *)(bs + 4);                                // 4 x 16 partial errors
    float *thr = (float *)(red + 64);                                // 16 thresholds (labels)
    int *thl = (int *)(thr + 16);                                    // 16 labels + count

    const int tid = threadIdx.x, nth = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwave = nth >> 6;
    const long long row = blockIdx.x;
    const float *Wr = prm.W + row * prm.ld;
    const float *Sr = prm.S + row * prm.ld;

    // ---- load, scale, encode ------------------------------------------------
    for (int j = tid; j < P; j += nth) {
        u64 key = ~0ull;
        if (j < m) {
            float wt, st;
            scaled_pair(Wr[j], Sr[j], prm.alpha, j, wt, st);
            if (st == 0.0f) st = 0.0f;
            key = ((u64)w_to_key(wt) << 32) | (u64)__float_as_uint(st);
        }
        sorted[swz((uint32_t)j)] = key;
    }
    if (tid < 4) bs[tid].active = 0;
    __syncthreads();

    // ---- sort by (w~, s~) ---------------------------------------------------
    sort_row(sorted, prm.logP, (uint32_t)tid);

    // ---- prefix sums of s~ and s~ w~ in sorted order -----------------------
    double total = 0.0;
    for (int pass = 0; pass < 2; ++pass) {
        double c = 0.0, q = 0.0;
        if (tid < nchunkP) {
            for (int e = 0; e < EPT; ++e) {
                const int r = tid * EPT + e;
                if (r < m) {
                    const u64 el = sorted[swz((uint32_t)r)];
                    const double s = (double)elem_s(el), w = (double)elem_w(el);
                    c += s;
                    q = fma(s, w, q);
                }
            }
            csum[tid] = make_double2(c, q);
        }
        {   // 256-element block sums: 16 neighbouring chunks
            double bc = c, bq = q;
            for (int d = 8; d >= 1; d >>= 1) {
                bc += __shfl_down(bc, d, 16);
                bq += __shfl_down(bq, d, 16);
            }
            if ((lane & 15) == 0 && tid < nchunkP) bsum[tid >> 4] = make_double2(bc, bq);
        }
        // running sum of s over the chunks (for the weighted-quantile start)
        double ic = c;
        for (int d = 1; d < 64; d <<= 1) {
            const double uc = __shfl_up(ic, d, 64);
            if (lane >= d) ic += uc;
        }
        if (lane == 63) wtot[wave] = ic;
        __syncthreads();
        if (wave == 0) {
            const double t = (lane < nwave) ? wtot[lane] : 0.0;
            double sc = t;
            for (int d = 1; d < 16; d <<= 1) {
                const double uc = __shfl_up(sc, d, 64);
                if (lane >= d) sc += uc;
            }
            if (lane < nwave) wtot[lane] = sc - t;  // exclusive
            if (lane == nwave - 1) wtot[16] = sc;
        }
        __syncthreads();
        {
            double xc = __shfl_up(ic, 1, 64);
            if (lane == 0) xc = 0.0;
            if (tid < nchunkP) cpre[tid] = wtot[wave] + xc;
        }
        total = wtot[16];
        if (tid == 0) cpre[nchunkP] = total;
        __syncthreads();
        if (total != 0.0 || pass == 1) break;
        // no sensitivity mass in this row: cluster with unit weights
        for (int j = tid; j < m; j += nth) {
            const uint32_t a = swz((uint32_t)j);
            sorted[a] = (sorted[a] & 0xFFFFFFFF00000000ull) | 0x3F800000ull;
        }
        __syncthreads();
    }

    // ---- Lloyd: one wavefront per bit width --------------------------------
    const int rowbits = prm.bits ? (int)prm.bits[row] : 0;
    if (wave < 4) {
        const int b = wave + 1;
        const bool on = prm.bits ? (b == rowbits) : (b >= prm.bmin && b <= prm.bmax);
        if (on) {
            switch (b) {
                case 1: lloyd_wave<1>(sorted, csum, bsum, cpre, m, prm.iters, total, &bs[wave]); break;
                case 2: lloyd_wave<2>(sorted, csum, bsum, cpre, m, prm.iters, total, &bs[wave]); break;
                case 3: lloyd_wave<3>(sorted, csum, bsum, cpre, m, prm.iters, total, &bs[wave]); break;
                default: lloyd_wave<4>(sorted, csum, bsum, cpre, m, prm.iters, total, &bs[wave]); break;
            }
            if (lane == 0) bs[wave].active = 1;
        }
    }
    __syncthreads();

    // ---- epilogue: errors, centroids, bounds, labels -----------------------
    double e4[4] = {0.0, 0.0, 0.0, 0.0};
    if (tid < nchunkP && tid * EPT < m) {
        const int r0 = tid * EPT;
        u64 el[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) el[e] = sorted[swz((uint32_t)(r0 + e))];
        for (int bi = 0; bi < 4; ++bi) {
            if (!bs[bi].active) continue;
            const int K = 2 << bi;
            int p = 0;
            while (p + 1 < K && bs[bi].B[p + 1] <= r0) ++p;
            int nextB = bs[bi].B[p + 1];
            double c = bs[bi].cent[p];
            double acc = 0.0;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int r = r0 + e;
                if (r < m) {
                    while (r >= nextB) {
                        ++p;
                        nextB = bs[bi].B[p + 1];
                        c = bs[bi].cent[p];
                    }
                    const double d = (double)elem_w(el[e]) - c;
                    acc += (double)elem_s(el[e]) * d * d;
                }
            }
            e4[bi] = acc;
        }
    }
#pragma unroll
    for (int bi = 0; bi < 4; ++bi) {
        double x = e4[bi];
        for (int d = 32; d >= 1; d >>= 1) x += __shfl_down(x, d, 64);
        if (lane == 0) red[bi * 16 + wave] = x;
    }
    __syncthreads();

    const int nb = prm.bmax - prm.bmin + 1;
    if (wave < 4 && bs[wave].active) {
        const int bi = wave, b = wave + 1, K = 1 << b;
        double x = (lane < nwave) ? red[bi * 16 + lane] : 0.0;
        for (int d = 8; d >= 1; d >>= 1) x += __shfl_down(x, d, 64);
        long long obase;
        if (prm.bits) {
            if (lane == 0) prm.E[row] = x;
            obase = row * 16;
        } else {
            if (lane == 0) prm.E[row * nb + (b - prm.bmin)] = x;
            obase = row * prm.stride + ((1 << b) - (1 << prm.bmin));
        }
        if (lane < K) {
            const int p = lane;
            const int k = bs[bi].idx[p];
            const int b0 = bs[bi].B[p], b1 = bs[bi].B[p + 1];
            const float up = (b1 > b0) ? elem_w(sorted[swz((uint32_t)(b1 - 1))]) : -INFINITY;
            prm.cent[obase + k] = bs[bi].cent[p];
            if (prm.upper) prm.upper[obase + k] = up;
            if (prm.bits) {
                thr[p] = up;
                thl[p] = k;
            }
        } else if (prm.bits && lane < 16) {
            prm.cent[obase + lane] = 0.0;
            if (prm.upper) prm.upper[obase + lane] = -INFINITY;
        }
    }
    if (prm.bits && prm.labels) {
        __syncthreads();
        // label of a column: the cluster whose value range holds w~ (ranges are
        // disjoint and ordered by position; empty ones have upper = -inf)
        const int K = 1 << rowbits;
        float th[16];
        int tl[16];
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            th[p] = (p < K) ? thr[p] : -INFINITY;
            tl[p] = (p < K) ? thl[p] : 0;
        }
        uint8_t *Lr = prm.labels + row * (long long)m;
        for (int j = tid; j < m; j += nth) {
            float wt, st;
            scaled_pair(Wr[j], Sr[j], prm.alpha, j, wt, st);
            int lab = -1, last = 0;
#pragma unroll
            for (int p = 0; p < 16; ++p) {
                const bool nonempty = th[p] != -INFINITY;
                if (nonempty) last = tl[p];
                if (lab < 0 && nonempty && wt <= th[p]) lab = tl[p];
            }
            Lr[j] = (uint8_t)(lab < 0 ? last : lab);
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

size_t cluster_lds_bytes(int P) {
    const int nchunkP = P >> 4;
    size_t b = (size_t)P * 8 + (size_t)nchunkP * 16 + (size_t)((nchunkP + 15) >> 4) * 16 + (size_t)(nchunkP + 1) * 8 +
               17 * 8 + 4 * sizeof(BitState) + 64 * 8 + 16 * 4 + 17 * 4;
    return (b + 15) & ~(size_t)15;
}

skim_status launch_cluster(skim_ctx *ctx, ClusterParams &prm, int64_t n) {
    int logP = 4;
    while ((1 << logP) < prm.m) ++logP;
    if (logP < 8) logP = 8;  // at least 256 keys: keeps the four Lloyd wavefronts' thread count simple
    prm.logP = logP;
    prm.P = 1 << logP;
    int threads = prm.P / EPT;
    if (threads < MIN_THREADS) threads = MIN_THREADS;
    const size_t lds = cluster_lds_bytes(prm.P);
    if ((int64_t)lds > ctx->lds_limit)
        SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "row length %d needs %zu bytes of LDS, device allows %d", prm.m, lds, ctx->lds_limit);
    static size_t lds_enabled = 0;
    if (lds > 65536 && lds > lds_enabled) {
        SKIM_HIP(ctx, hipFuncSetAttribute((const void *)cluster_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)ctx->lds_limit));
        lds_enabled = (size_t)ctx->lds_limit;
    }
    if (n == 0) return SKIM_OK;
    hipLaunchKernelGGL(cluster_kernel, dim3((unsigned)n), dim3(threads), lds, ctx->stream, prm);
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
    if (!centroids_all) {
        skim_ws_cursor cur{(char *)ctx->ws, 0, ctx->ws_bytes};
        centroids_all = (double *)cur.take((size_t)n * prm.stride * sizeof(double));
        if (!centroids_all) SKIM_FAIL(ctx, SKIM_ERR_WORKSPACE, "workspace too small for the centroid scratch");
    }
    prm.cent = centroids_all; prm.upper = upper_all; prm.labels = nullptr;
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
    return launch_cluster(ctx, prm, n);
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
