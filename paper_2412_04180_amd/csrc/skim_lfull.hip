// Error pre-recording with the layer-wise error (Alg. 3, pre-recording loop with Err(.) in its L-full
// form, Sec. 3.4 and the remark under Alg. 1): for every bit width the rows are clustered as
// in skim_error_table, each weight gets the label of its cluster, and the error of channel i
// is dW_i H dW_i^T.  Composition of the clustering call, a label kernel and the layer-loss
// kernels; one contraction dW * H per bit width.
#include "skim_common.h"

#include <math.h>

namespace {

constexpr int LAB_THREADS = 256;

// labels[i][j] = cluster of w~_ij at bit width b, from the clusters' upper bounds (the largest
// member of each cluster, -inf for an empty one): the cluster with the smallest bound >= w~.
__global__ void __launch_bounds__(LAB_THREADS) labels_from_bounds_kernel(const float *W, const float *alpha, long long m,
                                                                       long long ld, int K, const float *upper_all,
                                                                       int stride, int block_off, uint8_t *labels) {
    __shared__ float thr[16];
    __shared__ int thl[16];
    const long long row = blockIdx.x;
    const int tid = threadIdx.x;
    const float *up_row = upper_all + row * stride + block_off;
    if (tid < 16) {
        thr[tid] = INFINITY;
        thl[tid] = 0;
    }
    __syncthreads();
    if (tid < K) {
        const float up = up_row[tid];
        int rank = 0;
        for (int j = 0; j < K; ++j) {
            const float uj = up_row[j];
            rank += (uj < up || (uj == up && j < tid)) ? 1 : 0;
        }
        thr[rank] = up;
        thl[rank] = tid;
    }
    __syncthreads();
    // bounds ascending (empty clusters, -inf, first), +inf beyond the K-th
    if (tid >= K && tid < 16) thl[tid] = thl[K - 1];
    __syncthreads();
    const float *Wr = W + row * ld;
    uint8_t *Lr = labels + row * m;
    for (long long j = tid; j < m; j += LAB_THREADS) {
        const float w = Wr[j];
        const float wt = alpha ? __fdiv_rn(w, alpha[j]) : w;
        int pos = (thr[7] < wt) ? 8 : 0;
        pos += (thr[pos + 3] < wt) ? 4 : 0;
        pos += (thr[pos + 1] < wt) ? 2 : 0;
        pos += (thr[pos] < wt) ? 1 : 0;
        Lr[j] = (uint8_t)thl[pos];
    }
}

}  // namespace

extern "C" skim_status skim_error_table_lfull(skim_ctx *ctx, const float *W, const float *S, const float *alpha,
                                              const float *H, int64_t n, int64_t m, int64_t ld, int bmin, int bmax,
                                              int iters, double *E_full, double *E_sdiag, double *centroids_all,
                                              float *upper_all, uint8_t *labels_work) {
    skim_status st = skim_enter(ctx);
    if (st != SKIM_OK) return st;
    if (!W || !S || !H || !E_full || !centroids_all || !upper_all || !labels_work)
        SKIM_FAIL(ctx, SKIM_ERR_ARG, "skim_error_table_lfull: W, S, H, E_full, centroids_all, upper_all, labels_work must not be NULL");
    if (bmin < 1 || bmax > SKIM_MAX_BITS || bmin > bmax) SKIM_FAIL(ctx, SKIM_ERR_ARG, "bit range [%d,%d] outside 1..4", bmin, bmax);
    if (n < 1) SKIM_FAIL(ctx, SKIM_ERR_SHAPE, "n = %lld out of range", (long long)n);
    if (ctx->ws_bytes < skim_workspace_bytes(n, m))
        SKIM_FAIL(ctx, SKIM_ERR_WORKSPACE, "workspace missing or smaller than skim_workspace_bytes(n, m)");
    const int nb = bmax - bmin + 1;
    // the tail of the workspace holds what must survive the calls below (they carve from its start)
    const size_t tail_bytes = (((size_t)n * nb * sizeof(double) + 255) & ~(size_t)255) + 256;
    char *tail = (char *)ctx->ws + ((ctx->ws_bytes - tail_bytes) & ~(size_t)255);
    double *loss_scalar = (double *)tail;
    double *sdiag = E_sdiag ? E_sdiag : (double *)(tail + 256);
    if ((st = skim_error_table(ctx, W, S, alpha, n, m, ld, bmin, bmax, iters, sdiag, centroids_all, upper_all)) != SKIM_OK)
        return st;
    const int stride = (2 << bmax) - (1 << bmin);
    for (int b = bmin; b <= bmax; ++b) {
        hipLaunchKernelGGL(labels_from_bounds_kernel, dim3((unsigned)n), dim3(LAB_THREADS), 0, ctx->stream, W, alpha,
                           (long long)m, (long long)ld, 1 << b, upper_all, stride, (1 << b) - (1 << bmin), labels_work);
        SKIM_HIP(ctx, hipGetLastError());
        // a cluster whose members carry no sensitivity mass keeps the centroid the clustering left it with
        // (the value the packed codebook holds), not the 0 a weighted mean over no mass would give
        if ((st = skim_layer_loss_strided(ctx, W, S, alpha, H, n, m, ld, labels_work, loss_scalar, E_full + (b - bmin),
                                          nb, centroids_all + ((1 << b) - (1 << bmin)), stride, 1 << b)) != SKIM_OK)
            return st;
    }
    return SKIM_OK;
}
