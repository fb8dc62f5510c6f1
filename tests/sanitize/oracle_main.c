/* Drives every exported function of oracle/skim_oracle.c on small inputs (ragged lengths, a row without
 * mass, m == K, duplicates) so that AddressSanitizer and UndefinedBehaviorSanitizer see each code path.
 * Built and run by tests/test_sanitizers.py; prints "ok" when nothing fired.  Test infrastructure.        */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/skim_oracle.c"

static uint64_t rng_state = 12345;
static double uni(void) {
    rng_state = rng_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}
static double gauss(void) { return sqrt(-2.0 * log(uni() + 1e-300)) * cos(6.283185307179586 * uni()); }

static int run_case(int64_t n, int64_t m, int64_t ld, int with_alpha) {
    float *W = (float *)malloc((size_t)(n * ld) * sizeof(float));
    float *S = (float *)malloc((size_t)(n * ld) * sizeof(float));
    float *alpha = (float *)malloc((size_t)m * sizeof(float));
    for (int64_t i = 0; i < n * ld; ++i) {
        W[i] = (float)(0.02 * gauss());
        const double g = gauss();
        S[i] = (float)(g * g);
        if (uni() < 0.1 && i > 0) W[i] = W[i - 1];
        if (uni() < 0.1) S[i] = 0.0f;
    }
    if (n > 1)
        for (int64_t j = 0; j < m; ++j) S[ld + j] = 0.0f;   /* a row without mass */
    for (int64_t j = 0; j < m; ++j) alpha[j] = (float)exp(0.1 * gauss());
    const float *al = with_alpha ? alpha : NULL;
    int bmax = 4;
    while ((1 << bmax) > m) --bmax;
    const int nb = bmax;
    int stride = 0;
    for (int b = 1; b <= bmax; ++b) stride += 1 << b;
    double *E = (double *)malloc((size_t)(n * nb) * sizeof(double));
    double *ca = (double *)malloc((size_t)(n * stride) * sizeof(double));
    double *ua = (double *)malloc((size_t)(n * stride) * sizeof(double));
    int64_t near[2] = {0, 0};
    int64_t *near_rows = (int64_t *)calloc((size_t)n, sizeof(int64_t));
    int64_t *near_rb = (int64_t *)calloc((size_t)(n * nb), sizeof(int64_t));
    int rc = oracle_error_table(W, S, al, n, m, ld, 1, bmax, 30, E, ca, ua, near, near_rows, near_rb);
    if (rc) return rc;
    uint8_t *bits = (uint8_t *)malloc((size_t)n);
    int64_t spent, budget, gnear = 0;
    rc = oracle_greedy(E, NULL, n, 1, bmax, 0.5 * (1 + bmax), bits, &spent, &budget, &gnear);
    if (rc) return rc;
    int64_t *cost = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    for (int64_t i = 0; i < n; ++i) cost[i] = 1 + (i % 3);
    rc = oracle_greedy(E, cost, n, 1, bmax, 0.5 * (1 + bmax), bits, &spent, &budget, NULL);
    if (rc) return rc;
    uint8_t *labels = (uint8_t *)malloc((size_t)(n * m));
    double *cent = (double *)malloc((size_t)n * 16 * sizeof(double));
    double *upper = (double *)malloc((size_t)n * 16 * sizeof(double));
    double *err = (double *)malloc((size_t)n * sizeof(double));
    rc = oracle_cluster_rows(W, S, al, n, m, ld, bits, 30, labels, cent, upper, err, near_rows);
    if (rc) return rc;
    int64_t words = 0;
    for (int64_t i = 0; i < n; ++i) words += (m * bits[i] + 31) / 32;
    uint32_t *codes = (uint32_t *)malloc((size_t)(words + 1) * sizeof(uint32_t));
    int64_t gwo[6];
    int32_t *perm = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    uint16_t *cbs = (uint16_t *)malloc((size_t)n * 16 * sizeof(uint16_t));
    float *dW = (float *)malloc((size_t)(n * m) * sizeof(float));
    if (oracle_pack(W, al, n, m, ld, bits, labels, cent, codes, gwo, perm, cbs, dW) != words) return -100;
    double *c2 = (double *)malloc((size_t)n * 16 * sizeof(double));
    double *Den = (double *)malloc((size_t)n * 16 * sizeof(double));
    rc = oracle_centroids_from_labels(W, S, al, n, m, ld, labels, c2, Den);
    if (rc) return rc;
    float *H = (float *)malloc((size_t)(m * m) * sizeof(float));
    for (int64_t j = 0; j < m; ++j)
        for (int64_t l = 0; l <= j; ++l) H[j * m + l] = H[l * m + j] = (float)((j == l) ? 1.0 + uni() : 0.01 * gauss());
    double loss, *row_loss = (double *)malloc((size_t)n * sizeof(double));
    double *P = (double *)malloc((size_t)(n * m) * sizeof(double));
    rc = oracle_layer_loss(W, al, H, n, m, ld, labels, c2, &loss, row_loss, P);
    if (rc) return rc;
    rc = oracle_layer_loss(W, al, H, n, m, ld, labels, c2, &loss, NULL, NULL);
    if (rc) return rc;
    double *grad = (double *)malloc((size_t)m * sizeof(double));
    rc = oracle_scale_grad(W, S, alpha, H, n, m, ld, labels, &loss, grad, c2);
    if (rc) return rc;
    float *m1 = (float *)calloc((size_t)m, sizeof(float)), *m2 = (float *)calloc((size_t)m, sizeof(float));
    rc = oracle_adam_step(alpha, m1, m2, grad, m, 41, 0.01, 0.9, 0.999, 1e-8, 0.5, 40);
    if (rc) return rc;
    double c0[16];
    int64_t ranks[16];
    rc = oracle_quantile_init(W, S, m, 1 << bmax, c0, ranks);
    if (rc) return rc;
    free(m2); free(m1); free(grad); free(P); free(row_loss); free(H); free(Den); free(c2); free(dW); free(cbs);
    free(perm); free(codes); free(err); free(upper); free(cent); free(labels); free(cost); free(bits);
    free(near_rb); free(near_rows); free(ua); free(ca); free(E); free(alpha); free(S); free(W);
    return 0;
}

int main(void) {
    const int64_t shapes[][3] = {{1, 16, 16}, {3, 17, 20}, {5, 64, 64}, {4, 100, 128}, {2, 2, 2}, {7, 333, 333}, {2, 5, 9}};
    for (size_t k = 0; k < sizeof(shapes) / sizeof(shapes[0]); ++k)
        for (int a = 0; a < 2; ++a) {
            const int rc = run_case(shapes[k][0], shapes[k][1], shapes[k][2], a);
            if (rc) {
                printf("case %zu alpha %d failed with %d\n", k, a, rc);
                return 1;
            }
        }
    for (uint32_t h = 0; h < 65536; h += 7) {
        const float f = oracle_f16_to_f32((uint16_t)h);
        if (f == f && oracle_f32_to_f16(f) != (uint16_t)h) return 2;
    }
    printf("ok\n");
    return 0;
}
