/*
 * SKIM hot-path ORACLE  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what the hot path of SKIM
 * (arXiv 2412.04180) computes.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header,
 * table or helper with the HIP library and is never a fallback for it.
 *
 * Conventions
 *   W, S      row-major float32, n rows (output channels) of m weights, row
 *             stride ld elements.  S is the per-weight sensitivity (the
 *             paper's "Gradient Square" G, Alg. 3 input; Eq. S-diag in Sec. 3.3).
 *   alpha     optional column scaling vector (Sec. 4.3); NULL means all ones.
 *   all arithmetic is IEEE double on float inputs widened exactly, loops in
 *   natural index order, no blocking, no sorting inside the Lloyd loop.
 *
 * Each function names the passage of the paper it follows.  Where the paper
 * is silent the reading taken is stated next to the code.
 *
 * Parity pins (tests/test_oracle_*.py): exact 1-D K-means by dynamic
 * programming, numpy's weighted inverted-CDF quantile, closed forms for K=1
 * and m==K, power-of-two scale symmetries, brute-force allocation search,
 * an independent bit-stream unpacker, numpy float16 conversion, Frobenius /
 * diagonal / X-form identities for the layer loss, central finite differences
 * for the scale gradient and torch.optim.Adam for the optimiser step.
 */
#define _GNU_SOURCE
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_SHAPE (-2)
#define ORACLE_ERR_BUDGET (-3)

#define NEAR_TIE_REL 1e-9
#define KMAX 256

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Column scaling before clustering (Sec. 4.3: W^q = Quant(W * alpha^-1) * alpha).
 * Reading: the clustered values are w~ = fl32(w / alpha) and the K-means
 * weights become s~ = fl32(fl32(s * alpha) * alpha), the change of variables
 * under which sum s~ (w~ - c)^2 equals the S-diag objective on the
 * reconstructed weight alpha * c.  Both are single-precision IEEE operations
 * so that the clustering consumes float32 exactly like the unscaled case.   */
void oracle_scale_row(const float *w, const float *s, const float *alpha, int64_t m,
                      float *wt, float *st) {
    for (int64_t j = 0; j < m; ++j) {
        if (alpha) {
            volatile float q = w[j] / alpha[j];
            volatile float t = s[j] * alpha[j];
            volatile float u = t * alpha[j];
            wt[j] = q;
            st[j] = u;
        } else {
            wt[j] = w[j];
            st[j] = s[j];
        }
    }
}

/* ------------------------------------------------------------------ */
typedef struct {
    double w, s;
    int64_t j;
} elem_t;

static int cmp_elem(const void *pa, const void *pb) {
    const elem_t *a = (const elem_t *)pa, *b = (const elem_t *)pb;
    if (a->w < b->w) return -1;
    if (a->w > b->w) return 1;
    if (a->s < b->s) return -1;
    if (a->s > b->s) return 1;
    return (a->j > b->j) - (a->j < b->j);
}

/* Weighted-quantile initialisation (the Kmeans call of Alg. 3
 * does not say how centroids start; the workload definition fixes a
 * weighted-quantile start).  Reading:
 *   order the row ascending by (w, s, index); C_r = running sum of s in that
 *   order; centroid k starts at the element whose rank is the first r with
 *   C_r >= total * (2k+1) / (2K).  Ranks are then forced to be strictly
 *   increasing and to leave room for the remaining centroids, so the K
 *   starting points are K different elements of the row:
 *       r_k = min( max(raw_k, r_{k-1} + 1), m - K + k ).
 * s must already be the effective weights (unit weights if the row's total
 * sensitivity is zero).  near[0] counts rank decisions whose margin
 * |C_r - tau| / total is below 1e-9 at the chosen or the preceding rank.    */
static void quantile_init(const float *w, const double *s, int64_t m, int K, double *c0,
                          int64_t *ranks, int64_t *near) {
    elem_t *e = (elem_t *)malloc((size_t)m * sizeof(elem_t));
    double *C = (double *)malloc((size_t)m * sizeof(double));
    for (int64_t j = 0; j < m; ++j) {
        e[j].w = (double)w[j];
        e[j].s = s[j];
        e[j].j = j;
    }
    qsort(e, (size_t)m, sizeof(elem_t), cmp_elem);
    double run = 0.0;
    for (int64_t r = 0; r < m; ++r) {
        run += e[r].s;
        C[r] = run;
    }
    const double total = C[m - 1];
    int64_t prev = -1;
    for (int k = 0; k < K; ++k) {
        const double tau = total * (double)(2 * k + 1) / (double)(2 * K);
        int64_t raw = m - 1;
        for (int64_t r = 0; r < m; ++r) {
            if (C[r] >= tau) {
                raw = r;
                break;
            }
        }
        if (near) {
            int hit = fabs(C[raw] - tau) < NEAR_TIE_REL * total;
            if (raw > 0 && fabs(C[raw - 1] - tau) < NEAR_TIE_REL * total) hit = 1;
            if (hit) near[0] += 1;
        }
        int64_t r = raw;
        if (r < prev + 1) r = prev + 1;
        if (r > m - K + k) r = m - K + k;
        c0[k] = e[r].w;
        if (ranks) ranks[k] = r;
        prev = r;
    }
    free(C);
    free(e);
}

/* exported for the init pin */
int oracle_quantile_init(const float *w, const float *s, int64_t m, int K, double *c0,
                         int64_t *ranks) {
    if (m < K || K < 1 || K > KMAX) return ORACLE_ERR_SHAPE;
    double *sd = (double *)malloc((size_t)m * sizeof(double));
    double tot = 0.0;
    for (int64_t j = 0; j < m; ++j) {
        sd[j] = (double)s[j];
        tot += sd[j];
    }
    if (tot == 0.0)
        for (int64_t j = 0; j < m; ++j) sd[j] = 1.0;
    quantile_init(w, sd, m, K, c0, ranks, NULL);
    free(sd);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* One row of sensitivity-weighted 1-D K-means: Kmeans(W_i, weights = G_i,
 * n_centroids = 2^b) of the Kmeans call of Alg. 3, minimising the S-diag objective
 * sum_j s_j (w_j - c_{a_j})^2 (Sec. 3.3).  Plain Lloyd iteration:
 *   (A) every weight goes to its nearest centroid, |w - c_k| in double,
 *       the lowest k winning equal distances;
 *   (U) every centroid becomes the s-weighted mean of its members; a centroid
 *       whose members carry no weight mass (or that has no member) is kept.
 * T iterations from the weighted-quantile start, single start, no tolerance
 * stop.  The loop leaves early only when (A) repeats the previous assignment,
 * from where every later iteration would reproduce the same state exactly.
 *
 * Outputs: labels of the last (A); centroids after the last (U);
 * err = sum_j s_j (w_j - c_{a_j})^2 with those two; upper[k] = largest member
 * of cluster k (-inf when empty); J[t] (optional) the objective after
 * iteration t+1.  A row whose sensitivities sum to zero is clustered with
 * unit weights.
 * near (optional): near[0] += init near-ties, near[1] += assignment decisions
 * whose two best distances to value-distinct centroids differ by less than
 * 1e-9 * max_j |w_j|.                                                        */
int oracle_cluster_row(const float *w, const float *s, int64_t m, int K, int T, uint8_t *labels,
                       double *centroids, double *upper, double *err, double *J, int64_t *near) {
    if (K < 1 || K > KMAX || m < K || T < 1) return ORACLE_ERR_SHAPE;
    double *sd = (double *)malloc((size_t)m * sizeof(double));
    uint8_t *a = (uint8_t *)malloc((size_t)m);
    uint8_t *aprev = (uint8_t *)malloc((size_t)m);
    double c[KMAX], D[KMAX], N[KMAX];
    double total = 0.0, R = 0.0;
    for (int64_t j = 0; j < m; ++j) {
        sd[j] = (double)s[j];
        total += sd[j];
        double aw = fabs((double)w[j]);
        if (aw > R) R = aw;
    }
    if (total == 0.0)
        for (int64_t j = 0; j < m; ++j) sd[j] = 1.0;

    quantile_init(w, sd, m, K, c, NULL, near);

    double Jt = 0.0;
    int t = 0;
    for (; t < T; ++t) {
        /* (A) assignment */
        for (int64_t j = 0; j < m; ++j) {
            const double x = (double)w[j];
            int best = 0;
            double dbest = fabs(x - c[0]);
            for (int k = 1; k < K; ++k) {
                const double d = fabs(x - c[k]);
                if (d < dbest) {
                    dbest = d;
                    best = k;
                }
            }
            a[j] = (uint8_t)best;
            if (near) {
                double d2 = INFINITY;
                for (int k = 0; k < K; ++k) {
                    if (c[k] == c[best]) continue;
                    const double d = fabs(x - c[k]);
                    if (d < d2) d2 = d;
                }
                if (d2 - dbest < NEAR_TIE_REL * R) near[1] += 1;
            }
        }
        if (t > 0 && memcmp(a, aprev, (size_t)m) == 0) break; /* fixed point */
        /* (U) update */
        for (int k = 0; k < K; ++k) D[k] = N[k] = 0.0;
        for (int64_t j = 0; j < m; ++j) {
            D[a[j]] += sd[j];
            N[a[j]] += sd[j] * (double)w[j];
        }
        for (int k = 0; k < K; ++k)
            if (D[k] > 0.0) c[k] = N[k] / D[k];
        Jt = 0.0;
        for (int64_t j = 0; j < m; ++j) {
            const double d = (double)w[j] - c[a[j]];
            Jt += sd[j] * d * d;
        }
        if (J) J[t] = Jt;
        memcpy(aprev, a, (size_t)m);
    }
    if (J)
        for (int u = t; u < T; ++u) J[u] = Jt;

    for (int k = 0; k < K; ++k) {
        centroids[k] = c[k];
        if (upper) upper[k] = -INFINITY;
    }
    for (int64_t j = 0; j < m; ++j) {
        if (labels) labels[j] = aprev[j];
        if (upper && (double)w[j] > upper[aprev[j]]) upper[aprev[j]] = (double)w[j];
    }
    *err = Jt;
    free(aprev);
    free(a);
    free(sd);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Error pre-recording, Alg. 3, pre-recording loop: E[i][b - bmin] for every row and
 * every candidate bit width.  Reading: the recorded error is the S-diag
 * objective the clustering itself minimises (it needs only W and S); the
 * L-full error of the same clustering is what oracle_layer_loss returns per
 * row.  centroids_all / upper_all hold, per row, the blocks for b = bmin..bmax
 * back to back (2^bmin + ... + 2^bmax entries).  near: [0] init, [1] assign;
 * near_rows (optional, n entries): near-tie count of each row over all b;
 * near_rb (optional, n x nb): the same count per row and bit width.           */
int oracle_error_table(const float *W, const float *S, const float *alpha, int64_t n, int64_t m,
                       int64_t ld, int bmin, int bmax, int T, double *E, double *centroids_all,
                       double *upper_all, int64_t *near, int64_t *near_rows, int64_t *near_rb) {
    if (bmin < 1 || bmax > 8 || bmin > bmax) return ORACLE_ERR_ARG;
    if (m < (1 << bmax) || ld < m) return ORACLE_ERR_SHAPE;
    const int nb = bmax - bmin + 1;
    int stride = 0;
    for (int b = bmin; b <= bmax; ++b) stride += 1 << b;
    int64_t near0 = 0, near1 = 0;
    int rc = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 4) reduction(+ : near0, near1)
    for (int64_t i = 0; i < n; ++i) {
        float *wt = (float *)malloc((size_t)m * sizeof(float));
        float *st = (float *)malloc((size_t)m * sizeof(float));
        oracle_scale_row(W + i * ld, S + i * ld, alpha, m, wt, st);
        int off = 0;
        for (int b = bmin; b <= bmax; ++b) {
            const int K = 1 << b;
            double cbuf[KMAX], ubuf[KMAX], e;
            int64_t nt[2] = {0, 0};
            int r = oracle_cluster_row(wt, st, m, K, T, NULL, cbuf, ubuf, &e, NULL,
                                       (near || near_rows || near_rb) ? nt : NULL);
            if (r != ORACLE_OK) {
#pragma omp critical
                rc = r;
            }
            if (near_rows) near_rows[i] = (b == bmin ? 0 : near_rows[i]) + nt[0] + nt[1];
            if (near_rb) near_rb[i * nb + (b - bmin)] = nt[0] + nt[1];
            E[i * nb + (b - bmin)] = e;
            if (centroids_all) memcpy(centroids_all + i * stride + off, cbuf, sizeof(double) * K);
            if (upper_all) memcpy(upper_all + i * stride + off, ubuf, sizeof(double) * K);
            off += K;
            near0 += nt[0];
            near1 += nt[1];
        }
        free(st);
        free(wt);
    }
    if (near) {
        near[0] += near0;
        near[1] += near1;
    }
    return rc;
}

/* K-means at the allocated bit width of every row, Alg. 3, clustering loop at the allocated bits and the
 * re-clustering of W * alpha^-1 in Alg. 2.  centroids / upper are n x 16 with
 * the first 2^bits[i] entries of row i used (the rest set to 0 / -inf).
 * near_rows (optional, n entries) receives each row's near-tie count.         */
int oracle_cluster_rows(const float *W, const float *S, const float *alpha, int64_t n, int64_t m,
                        int64_t ld, const uint8_t *bits, int T, uint8_t *labels, double *centroids,
                        double *upper, double *err, int64_t *near_rows) {
    if (ld < m) return ORACLE_ERR_SHAPE;
    int rc = ORACLE_OK;
    for (int64_t i = 0; i < n; ++i)
        if (bits[i] < 1 || bits[i] > 4 || m < (1 << bits[i])) return ORACLE_ERR_SHAPE;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < n; ++i) {
        float *wt = (float *)malloc((size_t)m * sizeof(float));
        float *st = (float *)malloc((size_t)m * sizeof(float));
        oracle_scale_row(W + i * ld, S + i * ld, alpha, m, wt, st);
        const int K = 1 << bits[i];
        double cbuf[16], ubuf[16], e;
        int64_t nt[2] = {0, 0};
        int r = oracle_cluster_row(wt, st, m, K, T, labels ? labels + i * m : NULL, cbuf, ubuf, &e,
                                   NULL, near_rows ? nt : NULL);
        if (r != ORACLE_OK) {
#pragma omp critical
            rc = r;
        }
        for (int k = 0; k < 16; ++k) {
            centroids[i * 16 + k] = k < K ? cbuf[k] : 0.0;
            if (upper) upper[i * 16 + k] = k < K ? ubuf[k] : -INFINITY;
        }
        err[i] = e;
        if (near_rows) near_rows[i] = nt[0] + nt[1];
        free(st);
        free(wt);
    }
    return rc;
}

/* ------------------------------------------------------------------ */
/* Greedy bit allocation, Alg. 1.  Readings:
 *  - the row chosen at each step is the one with the largest error REDUCTION
 *    E[i][b_i] - E[i][b_i + 1] (the printed difference has the opposite sign,
 *    which would pick the least useful row of a minimisation problem);
 *  - the budget is B = floor(avg_bits * sum(cost) + 1e-9) bits and the loop
 *    stops when no still-upgradable row fits, so that the constraint
 *    (1/n) sum b_i <= avg_bits of Sec. 4.2 holds; with unit costs this is the
 *    stop rule of the listing (the bits handed out reach n times the target)
 *    whenever that product is an integer;
 *  - cost (optional) is the number of weights of each row, for tables that
 *    join matrices of different widths; the row maximising reduction / cost
 *    is taken.  NULL means unit cost, the algorithm as printed.
 *  Equal maxima: lowest row index.  near counts steps whose two best
 *  densities differ by less than 1e-9 relative.                              */
int oracle_greedy(const double *E, const int64_t *cost, int64_t n, int bmin, int bmax,
                  double avg_bits, uint8_t *bits, int64_t *spent_out, int64_t *budget_out,
                  int64_t *near) {
    if (bmin < 1 || bmax < bmin || n < 1) return ORACLE_ERR_ARG;
    const int nb = bmax - bmin + 1;
    int64_t csum = 0;
    for (int64_t i = 0; i < n; ++i) csum += cost ? cost[i] : 1;
    const int64_t B = (int64_t)floor(avg_bits * (double)csum + 1e-9);
    if (B < bmin * csum || B > bmax * csum) return ORACLE_ERR_BUDGET;
    int64_t spent = bmin * csum;
    for (int64_t i = 0; i < n; ++i) bits[i] = (uint8_t)bmin;
    for (;;) {
        int64_t best = -1, second = -1;
        double gbest = 0.0, gsecond = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            if (bits[i] >= bmax) continue;
            const int64_t ci = cost ? cost[i] : 1;
            if (ci > B - spent) continue;
            const int col = bits[i] - bmin;
            const double g = (E[i * nb + col] - E[i * nb + col + 1]) / (double)ci;
            if (best < 0 || g > gbest) {
                second = best;
                gsecond = gbest;
                best = i;
                gbest = g;
            } else if (second < 0 || g > gsecond) {
                second = i;
                gsecond = g;
            }
        }
        if (best < 0) break;
        if (near && second >= 0) {
            double scale = fabs(gbest) > 1e-300 ? fabs(gbest) : 1e-300;
            if ((gbest - gsecond) / scale < NEAR_TIE_REL) near[0] += 1;
        }
        bits[best] += 1;
        spent += cost ? cost[best] : 1;
    }
    if (spent_out) *spent_out = spent;
    if (budget_out) *budget_out = B;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* float32 -> IEEE binary16, round to nearest even, bit level.             */
uint16_t oracle_f32_to_f16(float f) {
    uint32_t x;
    memcpy(&x, &f, 4);
    const uint32_t sign = (x >> 16) & 0x8000u;
    const uint32_t e = (x >> 23) & 0xffu;
    uint32_t man = x & 0x7fffffu;
    if (e == 0xffu) return (uint16_t)(sign | 0x7c00u | (man ? 0x200u : 0u));
    const int32_t E = (int32_t)e - 127 + 15;
    if (E >= 31) return (uint16_t)(sign | 0x7c00u);
    if (E <= 0) {
        if (E < -10) return (uint16_t)sign;
        man |= 0x800000u;
        const int shift = 14 - E;
        uint32_t h = man >> shift;
        const uint32_t rem = man & ((1u << shift) - 1u);
        const uint32_t half = 1u << (shift - 1);
        if (rem > half || (rem == half && (h & 1u))) h += 1;
        return (uint16_t)(sign | h);
    }
    uint32_t h = ((uint32_t)E << 10) | (man >> 13);
    const uint32_t rem = man & 0x1fffu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) h += 1;
    return (uint16_t)(sign | h);
}

float oracle_f16_to_f32(uint16_t h) {
    const uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    const uint32_t e = (h >> 10) & 0x1fu;
    const uint32_t man = h & 0x3ffu;
    double v;
    if (e == 0)
        v = ldexp((double)man, -24);
    else if (e == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexp((double)(man | 0x400u), (int)e - 25);
    float f = (float)v;
    uint32_t x;
    memcpy(&x, &f, 4);
    x |= sign;
    memcpy(&f, &x, 4);
    return f;
}

/* Packing (Sec. 4.2, last paragraph; App. D.2): rows of equal bit width are
 * gathered and stored together, centroids in lower precision (Sec. 5.4).
 * The paper gives no bit layout; the one used here:
 *   rows ordered by (bits ascending, row index ascending) -> row_perm[p] = i;
 *   a row of b bits takes ceil(m*b/32) 32-bit words; the label of column j
 *   sits at bit j*b of the row's little-endian bit stream (word = pos >> 5,
 *   shift = pos & 31, spilling into the next word), unused high bits zero;
 *   group_word_offset[b] (b = 1..4) = first word of the b-bit group,
 *   group_word_offset[5] = total words, group_word_offset[0] = 0;
 *   codebooks: in the same row order, 2^b binary16 values per row, entry k =
 *   f16(f32(centroid k)) (both roundings to nearest even);
 *   dW (optional, n x m in ORIGINAL row order) = fl32(w - alpha * f32(code
 *   book value)), one rounding (fused multiply-add).
 * Returns the number of words written, or a negative status.                */
int64_t oracle_pack(const float *W, const float *alpha, int64_t n, int64_t m, int64_t ld,
                    const uint8_t *bits, const uint8_t *labels, const double *centroids,
                    uint32_t *codes, int64_t *group_word_offset, int32_t *row_perm,
                    uint16_t *codebooks, float *dW) {
    int64_t word = 0, cb = 0, p = 0;
    group_word_offset[0] = 0;
    for (int b = 1; b <= 4; ++b) {
        group_word_offset[b] = word;
        const int64_t wpr = (m * b + 31) / 32;
        for (int64_t i = 0; i < n; ++i) {
            if (bits[i] != b) continue;
            row_perm[p++] = (int32_t)i;
            uint32_t *out = codes + word;
            for (int64_t q = 0; q < wpr; ++q) out[q] = 0;
            for (int64_t j = 0; j < m; ++j) {
                const uint32_t code = labels[i * m + j];
                if (code >> b) return ORACLE_ERR_ARG;
                const int64_t pos = j * b;
                const int sh = (int)(pos & 31);
                out[pos >> 5] |= code << sh;
                if (sh + b > 32) out[(pos >> 5) + 1] |= code >> (32 - sh);
            }
            for (int k = 0; k < (1 << b); ++k) {
                const uint16_t h = oracle_f32_to_f16((float)centroids[i * 16 + k]);
                codebooks[cb + k] = h;
            }
            if (dW) {
                for (int64_t j = 0; j < m; ++j) {
                    const float q = oracle_f16_to_f32(codebooks[cb + labels[i * m + j]]);
                    const float a = alpha ? alpha[j] : 1.0f;
                    dW[i * m + j] = fmaf(-a, q, W[i * ld + j]);
                }
            }
            cb += 1 << b;
            word += wpr;
        }
    }
    if (p != n) return ORACLE_ERR_ARG; /* some row had bits outside 1..4 */
    group_word_offset[5] = word;
    return word;
}

/* ------------------------------------------------------------------ */
/* calc_centroids(W * alpha^-1, L) of Alg. 2 / the centroid update in the training loop of Alg. 3: with the labels
 * fixed, centroid k of row i is the weighted mean of its members in the
 * scaled domain, c_ik = sum s~ w~ / sum s~ (0 when the cluster carries no
 * mass).  Den (optional) returns the denominators.  c, Den are n x 16.      */
int oracle_centroids_from_labels(const float *W, const float *S, const float *alpha, int64_t n,
                                 int64_t m, int64_t ld, const uint8_t *labels, double *c,
                                 double *Den) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float *wt = (float *)malloc((size_t)m * sizeof(float));
        float *st = (float *)malloc((size_t)m * sizeof(float));
        oracle_scale_row(W + i * ld, S + i * ld, alpha, m, wt, st);
        double D[16] = {0}, N[16] = {0};
        for (int64_t j = 0; j < m; ++j) {
            const int k = labels[i * m + j] & 15;
            D[k] += (double)st[j];
            N[k] += (double)st[j] * (double)wt[j];
        }
        for (int k = 0; k < 16; ++k) {
            c[i * 16 + k] = D[k] > 0.0 ? N[k] / D[k] : 0.0;
            if (Den) Den[i * 16 + k] = D[k];
        }
        free(st);
        free(wt);
    }
    return ORACLE_OK;
}

/* Layer-wise (L-full) error, Sec. 3.4 and Alg. 2 "loss = Err(W, W^q)":
 *   dW_ij = w_ij - alpha_j * c[i][L_ij]           (W^q = replace(c, L) * alpha)
 *   loss  = sum_i dW_i H dW_i^T = sum_i sum_j sum_l dW_ij H_jl dW_il,
 * H (m x m, row-major float32) standing for X X^T.  Naive loops in double.
 * c is n x 16 double (from oracle_centroids_from_labels or a clustering).
 * row_loss (optional) gets each row's quadratic form; P (optional, n x m
 * double) gets dW * H.                                                      */
int oracle_layer_loss(const float *W, const float *alpha, const float *H, int64_t n, int64_t m,
                      int64_t ld, const uint8_t *labels, const double *c, double *loss,
                      double *row_loss, double *P) {
    double total = 0.0;
    double *rl = row_loss ? row_loss : (double *)malloc((size_t)n * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double *d = (double *)malloc((size_t)m * sizeof(double));
        for (int64_t j = 0; j < m; ++j) {
            const double a = alpha ? (double)alpha[j] : 1.0;
            d[j] = (double)W[i * ld + j] - a * c[i * 16 + (labels[i * m + j] & 15)];
        }
        double acc_row = 0.0;
        for (int64_t j = 0; j < m; ++j) {
            /* H is symmetric in exact arithmetic; (dW H)_j is taken as written,
             * sum_l dW_il H_lj, walking column j of H. */
            double pj = 0.0;
            for (int64_t l = 0; l < m; ++l) pj += d[l] * (double)H[l * m + j];
            if (P) P[i * m + j] = pj;
            acc_row += pj * d[j];
        }
        rl[i] = acc_row;
        free(d);
    }
    for (int64_t i = 0; i < n; ++i) total += rl[i];
    if (!row_loss) free(rl);
    *loss = total;
    return ORACLE_OK;
}

/* Gradient of the layer loss with respect to alpha with the labels fixed and
 * the centroids recomputed from alpha (Alg. 2: c = calc_centroids(W*alpha^-1,
 * L) sits inside the training loop, so loss.backward() differentiates through
 * it).  With the effective weights s~ = s alpha^2 and values w~ = w / alpha:
 *   N_ik = sum_{j in k} s_ij alpha_j w_ij,  D_ik = sum_{j in k} s_ij alpha_j^2,
 *   c_ik = N_ik / D_ik,  dW_ij = w_ij - alpha_j c_{i,L_ij},  P = dW H,
 *   Q_ik = sum_{j in k} P_ij alpha_j  (H symmetric), and
 *   d loss / d alpha_l = -2 sum_i [ P_il c_{i,L_il}
 *                        + Q_{i,L_il} s_il (w_il - 2 alpha_l c_{i,L_il}) / D_{i,L_il} ].
 * The second term is dropped for clusters without mass.  Here c, N, D are
 * formed in double from the unrounded expressions above (the rounding of the
 * float32 w~, s~ used by the clustering is far below the gradient tolerance).
 * Also returns the loss and (optionally) the centroids used.                */
int oracle_scale_grad(const float *W, const float *S, const float *alpha, const float *H, int64_t n,
                      int64_t m, int64_t ld, const uint8_t *labels, double *loss, double *grad,
                      double *c_out) {
    double *c = (double *)calloc((size_t)n * 16 + 1, sizeof(double));
    double *Dn = (double *)malloc((size_t)n * 16 * sizeof(double));
    double *P = (double *)malloc((size_t)n * (size_t)m * sizeof(double));
    for (int64_t i = 0; i < n; ++i) {
        double N[16] = {0}, D[16] = {0};
        for (int64_t j = 0; j < m; ++j) {
            const int k = labels[i * m + j] & 15;
            const double a = alpha ? (double)alpha[j] : 1.0;
            const double s = (double)S[i * ld + j], w = (double)W[i * ld + j];
            N[k] += s * a * w;
            D[k] += s * a * a;
        }
        for (int k = 0; k < 16; ++k) {
            c[i * 16 + k] = D[k] > 0.0 ? N[k] / D[k] : 0.0;
            Dn[i * 16 + k] = D[k];
        }
    }
    oracle_layer_loss(W, alpha, H, n, m, ld, labels, c, loss, NULL, P);
    for (int64_t l = 0; l < m; ++l) grad[l] = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double Q[16] = {0};
        for (int64_t j = 0; j < m; ++j) {
            const double a = alpha ? (double)alpha[j] : 1.0;
            Q[labels[i * m + j] & 15] += P[i * m + j] * a;
        }
        for (int64_t l = 0; l < m; ++l) {
            const int k = labels[i * m + l] & 15;
            const double a = alpha ? (double)alpha[l] : 1.0;
            const double ck = c[i * 16 + k];
            double term = P[i * m + l] * ck;
            if (Dn[i * 16 + k] > 0.0)
                term += Q[k] * (double)S[i * ld + l] * ((double)W[i * ld + l] - 2.0 * a * ck) /
                        Dn[i * 16 + k];
            grad[l] += -2.0 * term;
        }
    }
    if (c_out) memcpy(c_out, c, (size_t)n * 16 * sizeof(double));
    free(P);
    free(Dn);
    free(c);
    return ORACLE_OK;
}

/* One Adam step on alpha (Sec. 5.1: Adam, learning rate 0.01 halved every 40
 * steps).  The paper gives no further constants; reading: beta1 = 0.9,
 * beta2 = 0.999, eps = 1e-8, bias-corrected moments (the optimiser's
 * published defaults), lr_t = lr0 * decay^floor((t-1)/decay_every), t >= 1.
 * State is float32; arithmetic here is double, stored back rounded.         */
int oracle_adam_step(float *alpha, float *m1, float *m2, const double *grad, int64_t m, int64_t t,
                     double lr0, double beta1, double beta2, double eps, double decay,
                     int64_t decay_every) {
    if (t < 1) return ORACLE_ERR_ARG;
    const double lr = lr0 * pow(decay, (double)((t - 1) / decay_every));
    const double bc1 = 1.0 - pow(beta1, (double)t), bc2 = 1.0 - pow(beta2, (double)t);
    for (int64_t j = 0; j < m; ++j) {
        const double g = grad[j];
        const double a = beta1 * (double)m1[j] + (1.0 - beta1) * g;
        const double v = beta2 * (double)m2[j] + (1.0 - beta2) * g * g;
        m1[j] = (float)a;
        m2[j] = (float)v;
        const double step = lr * (a / bc1) / (sqrt(v / bc2) + eps);
        alpha[j] = (float)((double)alpha[j] - step);
    }
    return ORACLE_OK;
}
