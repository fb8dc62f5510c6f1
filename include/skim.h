/*
 * skim.h -- C ABI of the MI355X (gfx950) implementation of the data-parallel
 * hot path of SKIM (arXiv 2412.04180): per-output-channel sensitivity-weighted
 * 1-D K-means at every candidate bit width, the channel x bit error table,
 * greedy mixed-precision bit allocation, packing, and the scaling-vector step
 * with its layer-wise loss.
 *
 * General rules
 *   - Plain C types only.  "dev" = pointer to device (HBM) memory of the
 *     context's GPU, "host" = pointer to host memory.
 *   - The caller owns every buffer.  The calls allocate no device memory:
 *     scratch comes from the workspace the caller registers (skim_create alone
 *     allocates 256 bytes that the context keeps until skim_destroy: the
 *     counters from which the row sort's workgroups take their rows).  The
 *     library keeps no pointer after a call returns, except the registered
 *     workspace.
 *   - Device calls enqueue work on the context's HIP stream and return without
 *     synchronising; results (including scalars) land in device memory.
 *     skim_greedy_allocate is synchronous host code.
 *   - Matrices are row-major; a row is one output channel.  ld is the row
 *     stride in elements (ld >= m).
 *   - Every call returns SKIM_OK or a negative skim_status; after an error the
 *     outputs are unspecified and skim_last_error() describes the cause.
 *     There is no CPU fallback: without a usable GPU, skim_create fails.
 *   - Inputs must be finite, S >= 0, alpha > 0.  Violations are not detected.
 *   - Calls on one context must not overlap in time (they share the workspace).
 *
 * Labels and cluster order.  Cluster k of a row (k = 0 .. 2^b - 1) is the k-th
 * starting centroid, taken at ascending weighted quantiles of the row; a
 * label is that cluster index.  Centroid values are almost always ascending in
 * k but the library does not rely on it.
 */
#ifndef SKIM_H
#define SKIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct skim_ctx skim_ctx;

typedef enum {
    SKIM_OK = 0,
    SKIM_ERR_ARG = -1,       /* null pointer, bit range, iteration count ...          */
    SKIM_ERR_SHAPE = -2,     /* n, m, ld outside what the kernels support               */
    SKIM_ERR_BUDGET = -3,    /* average bits outside [bmin, bmax]                       */
    SKIM_ERR_WORKSPACE = -4, /* workspace missing or too small                          */
    SKIM_ERR_HIP = -5,       /* a HIP runtime call failed                               */
    SKIM_ERR_NONFINITE = -6  /* validation on: W, S or alpha holds a value the method is undefined on */
} skim_status;

/* Adam with step decay for the scaling vector (Sec. 5.1 "Settings": Adam,
 * lr 0.01 halved every 40 steps).  beta1/beta2/eps are the optimiser's
 * published defaults 0.9 / 0.999 / 1e-8; moments are bias-corrected. */
typedef struct {
    float lr0, beta1, beta2, eps, decay;
    int32_t decay_every;
} skim_adam_opts;

#define SKIM_MAX_BITS 4
#define SKIM_MAX_K 16
/* Longest row the clustering accepts (rows up to 16384 weights are sorted in one
 * LDS pass, longer ones in two halves merged in global memory). */
#define SKIM_MAX_M 32768

/* ---- context ------------------------------------------------------------ */

/* Create a context on GPU `device` that enqueues on `hip_stream` (a
 * hipStream_t passed as void*, NULL = the default stream).  Fails with
 * SKIM_ERR_HIP when the device is not a usable gfx950 GPU.  Allocates the
 * context's 256 bytes of device memory and synchronises the device once;
 * not for use under stream capture. */
skim_status skim_create(skim_ctx **out, int device, void *hip_stream);
skim_status skim_destroy(skim_ctx *ctx);
/* Text of the last error on this context (ctx-owned, valid until the next
 * call); ctx == NULL returns the text of the last skim_create failure. */
const char *skim_last_error(const skim_ctx *ctx);

/* Scratch needed by any call on an n x m matrix (bytes), and its registration.
 * dev pointer, 256-byte aligned, must stay valid while calls use it. */
size_t skim_workspace_bytes(int64_t n, int64_t m);
skim_status skim_set_workspace(skim_ctx *ctx, void *dev_ptr, size_t bytes);

/* Optional validation of the inputs of the clustering calls (skim_error_table,
 * skim_cluster_rows and the calls built on them).  The method is undefined on
 * weights that are not finite, sensitivities that are negative or not finite
 * and scales that are not positive finite numbers; by default such inputs are
 * not looked for (the result is then unspecified, every access stays in
 * bounds).  With validation on, each such call first runs one pass over W, S
 * and alpha, waits for it (the call synchronises with the stream), and returns
 * SKIM_ERR_NONFINITE, with the text naming the array, before any other work.
 * Uses 256 bytes of the registered workspace. */
skim_status skim_validate_enable(skim_ctx *ctx, int on);

/* Optional timing of the two phases of a clustering call (skim_error_table,
 * skim_cluster_rows) with HIP events on the context's stream: the sort phase
 * (load, sort, sums) and the Lloyd phase (iterations, errors, outputs).
 * skim_profile_last synchronises on the last timed call and returns the two
 * durations in milliseconds (host pointers, may be NULL).  For benchmarks:
 * timing is off by default and adds nothing to untimed calls. */
skim_status skim_profile_enable(skim_ctx *ctx, int on);
skim_status skim_profile_last(skim_ctx *ctx, float *sort_ms, float *lloyd_ms);

/* ---- clustering --------------------------------------------------------- */

/* Error pre-recording (Alg. 3, pre-recording loop): for every row i and every bit
 * width b in [bmin, bmax] run the weighted K-means
 *     Kmeans(W_i * alpha^-1, weights = S_i * alpha^2, n_centroids = 2^b)
 * (the Kmeans call of Alg. 3; objective: the S-diag form of Sec. 3.3) from the
 * weighted-quantile start for `iters` Lloyd iterations and record
 *     E[i][b - bmin] = sum_j s~_ij (w~_ij - c_{a_ij})^2 .
 * W, S: dev, n x m float32, stride ld.  alpha: dev, m float32, or NULL (= 1).
 * E: dev, n x (bmax-bmin+1) float64.
 * centroids_all: dev float64, n x (2^bmin + ... + 2^bmax), per row the blocks
 *   for b = bmin..bmax back to back; may be NULL.
 * upper_all: dev float32, same layout: largest member w~ of each cluster,
 *   -inf for an empty cluster (the thresholds skim_pack rebuilds labels from);
 *   may be NULL.
 * 1 <= bmin <= bmax <= 4, 2^bmax <= m <= SKIM_MAX_M, iters >= 1. */
skim_status skim_error_table(skim_ctx *ctx, const float *W, const float *S, const float *alpha,
                             int64_t n, int64_t m, int64_t ld, int bmin, int bmax, int iters,
                             double *E, double *centroids_all, float *upper_all);

/* K-means at one bit width per row (Alg. 3, clustering loop at the allocated bits; the re-clustering of
 * W * alpha^-1 in Alg. 2).  bits: dev uint8[n], each in 1..4.
 * labels: dev uint8 n x m (dense, stride m), may be NULL.
 * centroids: dev float64 n x 16 (first 2^bits[i] used, rest 0).
 * upper: dev float32 n x 16 (rest -inf), may be NULL.  err: dev float64[n]. */
skim_status skim_cluster_rows(skim_ctx *ctx, const float *W, const float *S, const float *alpha,
                              int64_t n, int64_t m, int64_t ld, const uint8_t *bits, int iters,
                              uint8_t *labels, double *centroids, float *upper, double *err);

/* Pick, for every row, the block of its allocated bit width out of the
 * per-bit outputs of skim_error_table (clustering is deterministic, so the
 * K-means of Alg. 3, clustering loop at the allocated bits need not be run again).  All pointers dev.
 * centroids: n x 16 float64, upper: n x 16 float32 (layout of
 * skim_cluster_rows), err: float64[n], may be NULL. */
skim_status skim_select_allocated(skim_ctx *ctx, int64_t n, int bmin, int bmax, const uint8_t *bits,
                                  const double *E, const double *centroids_all,
                                  const float *upper_all, double *centroids, float *upper,
                                  double *err);

/* The least value of the clustering objective (the S-diag form, as in
 * skim_error_table) that ANY assignment of a row to at most 2^b clusters can
 * have, b = bmin..bmax: the floor under what the K-means of Alg. 3 reaches from
 * its start, a yardstick and not a step of the quantisation path.  In one
 * dimension the best assignment cuts the sorted values into intervals, which a
 * dynamic programme over the sorted row finds exactly (filled by halving, using
 * that the best cut moves right with the prefix).  Arguments as
 * skim_error_table (alpha may be NULL; a row without sensitivity mass counts
 * unit weights).  E_opt: dev float64 n x (bmax-bmin+1).  Costs are formed from
 * float64 prefix sums of s, s w, s w^2, so an entry carries an absolute error of
 * a few 1e-16 * sum_j s w^2 of its row.  scratch: dev, 256-byte aligned, at
 * least skim_kmeans_optimal_scratch_bytes(n, m) bytes (44 bytes per column and
 * resident workgroup); the registered workspace is used for the sort. */
size_t skim_kmeans_optimal_scratch_bytes(int64_t n, int64_t m);
skim_status skim_kmeans_optimal(skim_ctx *ctx, const float *W, const float *S, const float *alpha,
                                int64_t n, int64_t m, int64_t ld, int bmin, int bmax, double *E_opt,
                                void *scratch, size_t scratch_bytes);

/* ---- allocation --------------------------------------------------------- */

/* Greedy bit allocation (Alg. 1), host memory only.  E: host float64
 * n x (bmax-bmin+1).  Every row starts at bmin; the row with the largest error
 * reduction per unit cost, E[i][b_i] - E[i][b_i+1] over row_cost[i], gets one
 * more bit while it fits the budget floor(avg_bits * sum(cost) + 1e-9); equal
 * reductions go to the lowest row index.  row_cost: host int64[n] (weights per
 * row, for tables joining matrices of different width) or NULL = unit cost,
 * the algorithm as printed.  bits_out: host uint8[n].  spent_out, budget_out
 * (may be NULL): bits spent / available, in cost units. */
skim_status skim_greedy_allocate(const double *E, const int64_t *row_cost, int64_t n, int bmin,
                                 int bmax, double avg_bits, uint8_t *bits_out, int64_t *spent_out,
                                 int64_t *budget_out);

/* The same allocation with unit costs (Alg. 1 as printed) on the device: E, bits
 * dev pointers, launched on the context's stream, no synchronisation with the
 * host.  info: dev int64[10]: [b] = rows that got b bits (b = 0..7), [8] = bits
 * spent, [9] = budget.  Result identical to skim_greedy_allocate(row_cost = NULL).
 * Uses the start of the workspace (8 bytes per row and possible upgrade). */
skim_status skim_greedy_allocate_device(skim_ctx *ctx, const double *E, int64_t n, int bmin, int bmax,
                                        double avg_bits, uint8_t *bits, int64_t *info);

/* The exact optimum of the allocation problem that Alg. 1 approximates (the
 * bit-constrained sum minimisation stated with the mixed-precision problem,
 * which the paper notes a dynamic programme solves exactly): bits b_i in
 * [bmin, bmax], bmax - bmin <= 3, minimising sum_i E[i][b_i] subject to
 * sum_i b_i <= floor(avg_bits * n + 1e-9), unit costs.  A yardstick for the
 * greedy result, not a step of the quantisation path.  Rows are taken in
 * index order, f_{i+1}[x] = min_d f_i[x - d] + E[i][bmin + d] over the bits x
 * spent above bmin; equal sums keep the smaller d and the least final state
 * wins, so the result is a function of E alone.  E, bits: dev, as in
 * skim_greedy_allocate_device.  info: dev float64[3] = least total error, bits
 * spent, budget.  scratch: dev, 256-byte aligned, at least
 * skim_dp_allocate_scratch_bytes(...) bytes (about n * (budget - n * bmin)
 * bytes; 0 is returned for arguments the call would reject).  Launched on
 * the context's stream, no synchronisation with the host. */
size_t skim_dp_allocate_scratch_bytes(int64_t n, int bmin, int bmax, double avg_bits);
skim_status skim_dp_allocate(skim_ctx *ctx, const double *E, int64_t n, int bmin, int bmax,
                             double avg_bits, uint8_t *bits, double *info, void *scratch,
                             size_t scratch_bytes);

/* ---- packing ------------------------------------------------------------ */

/* Number of 32-bit words / binary16 codebook entries skim_pack writes for the
 * given host bits[n] (each 1..4). */
int64_t skim_packed_words(const uint8_t *bits_host, int64_t n, int64_t m);
int64_t skim_codebook_entries(const uint8_t *bits_host, int64_t n);

/* Pack (Sec. 4.2 last paragraph, App. D.2: rows of equal bit width are
 * gathered and processed together; Sec. 5.4: centroids in lower precision).
 * Layout: rows ordered by (bits ascending, row index ascending), row_perm[p] =
 * original row; a b-bit row takes ceil(m*b/32) uint32 words, the label of
 * column j at bit j*b of the row's little-endian bit stream, padding bits 0;
 * group_word_offset[b] (b=1..4) = first word of the b-bit group, [5] = total,
 * [0] = 0.  codebooks: same row order, 2^b binary16 per row,
 * f16(f32(centroid)) both round-to-nearest-even.  dW (optional, n x m float32,
 * stride m, original row order) = fl32(w - alpha * f32(codebook value)).
 * Labels are rebuilt from the thresholds: the cluster with the smallest upper
 * bound >= w~.  All pointers dev; group_word_offset is dev int64[6].
 * m < 2^29 (SKIM_ERR_SHAPE beyond). */
skim_status skim_pack(skim_ctx *ctx, const float *W, const float *alpha, int64_t n, int64_t m,
                      int64_t ld, const uint8_t *bits, const double *centroids, const float *upper,
                      uint32_t *codes, int64_t *group_word_offset, int32_t *row_perm,
                      uint16_t *codebooks_fp16, float *dW);

/* skim_pack for callers that cannot allocate device memory or hand over a
 * workspace (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): same arguments, same results, but the scratch of the call
 * (one int per row and a small group table) lives in a device array inside the
 * library instead of the workspace, so the call allocates nothing and needs no
 * skim_set_workspace.  n <= SKIM_PACK_STATIC_MAX_ROWS (SKIM_ERR_SHAPE beyond;
 * use skim_pack then).  Every GPU the library runs on holds its own copy of the
 * array (256 KiB) until the process ends; all calls on one GPU share it, so
 * calls that overlap on one GPU (different streams or threads) race -- issue
 * them on one stream.  Nothing in the array has to survive or be cleared
 * between calls: every call writes what it reads. */
#define SKIM_PACK_STATIC_MAX_ROWS 65536
skim_status skim_pack_static(skim_ctx *ctx, const float *W, const float *alpha, int64_t n, int64_t m,
                             int64_t ld, const uint8_t *bits, const double *centroids,
                             const float *upper, uint32_t *codes, int64_t *group_word_offset,
                             int32_t *row_perm, uint16_t *codebooks_fp16, float *dW);

/* ---- readers of the packed model ------------------------------------------ */

/* Dequantisation of what skim_pack wrote (same layout, dev pointers):
 *   Wq[i][j] = fl32(alpha_j * f32(codebook_i[code_ij]))   (alpha NULL: f32(codebook))
 * Wq: dev float32 n x m, stride m, original row order.  Rows whose bit width the
 * packed model does not hold (bits outside 1..4 at pack time) are not written. */
skim_status skim_unpack(skim_ctx *ctx, const uint32_t *codes, const int64_t *group_word_offset,
                        const int32_t *row_perm, const uint16_t *codebooks_fp16, const float *alpha,
                        int64_t n, int64_t m, float *Wq);

/* Matrix-vector product with the packed model, bit-width group by group, every
 * weight looked up in its row's binary16 codebook (the inference-side use of
 * the layout, Sec. 4.2 last paragraph, App. D.2):
 *   y[i] = sum_j Wq[i][j] * x[j],  Wq as above, products and sum in float64.
 * n = number of packed rows (group_word_offset and row_perm describe them).
 * x: dev float32[m].  y: dev float64, indexed by original row. */
skim_status skim_dequant_matvec(skim_ctx *ctx, const uint32_t *codes, const int64_t *group_word_offset,
                                const int32_t *row_perm, const uint16_t *codebooks_fp16,
                                const float *alpha, int64_t n, int64_t m, const float *x, double *y);

/* The same product in float32, for a reader bound by the packed bytes it
 * streams rather than by float64 arithmetic (the memory footprint argument of
 * Sec. 5.4 and the packed layout of App. D.2 are about this reader):
 *   y[i] = sum_j f32(codebook_i[code_ij]) * (alpha_j * x_j),  fused multiply-adds
 * in float32, a summation order of its own; it agrees with skim_dequant_matvec
 * to about 1e-6 of sum_j |Wq_ij x_j|.  y: dev float32, indexed by original row. */
skim_status skim_dequant_matvec_f32(skim_ctx *ctx, const uint32_t *codes, const int64_t *group_word_offset,
                                    const int32_t *row_perm, const uint16_t *codebooks_fp16,
                                    const float *alpha, int64_t n, int64_t m, const float *x, float *y);

/* ---- scaling vector ----------------------------------------------------- */

/* Layer-wise Hessian proxy from calibration activations (Sec. 3.4):
 *   H = X^T X / N,  X: dev N x m bfloat16 (bit patterns, row-major, one activation
 *   vector per row; 4-byte aligned, m even),  H: dev m x m float32.
 * bf16 MFMA with float32 accumulation over chunks of activations (2048; 8192 for
 * m > 2560 with m % 8 == 0, X 16-byte aligned and N >= 128, where the chunks are
 * added up in float32 in H itself and only the tiles on and above the diagonal are
 * computed; otherwise in float64); every entry within 1e-5 of sqrt(H_jj H_ll) for N up
 * to about 10^6; H comes out symmetric bit for bit.  H is written only (its
 * previous contents do not matter). */
skim_status skim_hessian_from_activations(skim_ctx *ctx, const uint16_t *X_bf16, int64_t N, int64_t m,
                                          float *H);

/* Layer-wise (L-full) loss of Alg. 2 with fixed labels:
 *   c   = calc_centroids(W * alpha^-1, L)      (weighted means, weights S alpha^2)
 *   dW  = W - replace(c, L) * alpha
 *   loss = tr(dW H dW^T) = sum_i dW_i H dW_i^T  (Sec. 3.4, L-full; H ~ X X^T)
 * H: dev m x m float32 (symmetric).  labels: dev uint8 n x m.  loss: dev
 * float64 scalar.  row_loss: dev float64[n] (the L-full error of each channel),
 * may be NULL.  The contraction dW*H accumulates in float32 on the matrix cores:
 * for m a multiple of 32 (and >= 128) on the bf16 ones, with every float32 operand
 * cut exactly into three bfloat16 pieces and the six leading piece products taken
 * per k (what is dropped is below 2^-24 of each product, the size of float32's own
 * rounding); otherwise on the fp32 ones.  The bf16 path reads row j of H for its
 * column j: H must be symmetric, as the H of Sec. 3.4 is.  The final reductions are
 * float64.  m must be a multiple of 16. */
skim_status skim_layer_loss(skim_ctx *ctx, const float *W, const float *S, const float *alpha,
                            const float *H, int64_t n, int64_t m, int64_t ld,
                            const uint8_t *labels, double *loss, double *row_loss);

/* Error pre-recording with the layer-wise error (Alg. 3, pre-recording loop, with the
 * error taken in its L-full form as Sec. 4.2 prescribes; Sec. 3.4): the rows are
 * clustered for every b in [bmin, bmax] exactly as in skim_error_table, and
 *   E_full[i][b-bmin] = dW_i H dW_i^T,  dW_i = w_i - alpha * c_{i, L_i}
 * with L the labels of that clustering and c the weighted means of its clusters
 * (a cluster whose members carry no sensitivity mass keeps the centroid the
 * clustering left it with, the value skim_pack stores; one contraction
 * dW * H per bit width as in skim_layer_loss, float64 reductions).
 * E_full: dev float64 n x nb.  E_sdiag: dev float64 n x nb, the S-diag errors
 * of the same clusterings (what skim_error_table returns), may be NULL.
 * centroids_all, upper_all: as in skim_error_table, required.  labels_work:
 * dev uint8 n x m scratch (holds the labels of the last bit width on return).
 * H: dev m x m float32, 16-byte aligned; m must be a multiple of 16 (the limits
 * of skim_layer_loss).  The workspace must hold skim_workspace_bytes(n, m). */
skim_status skim_error_table_lfull(skim_ctx *ctx, const float *W, const float *S, const float *alpha,
                                   const float *H, int64_t n, int64_t m, int64_t ld,
                                   int bmin, int bmax, int iters,
                                   double *E_full, double *E_sdiag, double *centroids_all,
                                   float *upper_all, uint8_t *labels_work);

/* One optimiser step on alpha with the labels fixed (inner loop of Alg. 2):
 * the loss above, its gradient with respect to alpha through the centroids,
 * and an Adam update of alpha / adam_m / adam_v (dev float32[m], in place).
 * t is the 1-based step number (selects the decayed learning rate and the bias
 * correction).  loss_before: dev float64 scalar (loss at the incoming alpha).
 * grad_out: dev float32[m], may be NULL. */
skim_status skim_scale_step(skim_ctx *ctx, const float *W, const float *S, const float *H,
                            int64_t n, int64_t m, int64_t ld, const uint8_t *labels, float *alpha,
                            float *adam_m, float *adam_v, int64_t t, const skim_adam_opts *opts,
                            double *loss_before, float *grad_out);

/* Scaling-vector training, Alg. 2 as a whole: `outer` rounds (the algorithm's I) of
 *   L = labels of Kmeans(W * alpha^-1) at the bit widths bits[i]   (skim_cluster_rows)
 *   `steps` optimiser steps on alpha with L fixed                    (skim_scale_step)
 * and on return c = calc_centroids(W * alpha^-1, L) at the final alpha.  The paper
 * trains until "converged" with at most 120 steps (Sec. 5.1); this call runs exactly
 * `steps` steps per round.  Step numbers (learning-rate decay, bias correction) run
 * t0, t0+1, ... across the rounds; alpha, adam_m, adam_v: dev float32[m], in/out.
 * labels: dev uint8 n x m (out), centroids: dev float64 n x 16 (out).
 * loss_trace: dev float64[outer*steps + 1]: the loss before every step, then the loss
 * at the returned alpha.  Limits of skim_layer_loss apply (m multiple of 16, H aligned). */
skim_status skim_train_scale(skim_ctx *ctx, const float *W, const float *S, const float *H,
                             int64_t n, int64_t m, int64_t ld, const uint8_t *bits,
                             int kmeans_iters, int outer, int steps, int64_t t0,
                             const skim_adam_opts *opts, float *alpha, float *adam_m, float *adam_v,
                             uint8_t *labels, double *centroids, double *loss_trace);

#ifdef __cplusplus
}
#endif
#endif /* SKIM_H */
