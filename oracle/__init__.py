"""ctypes front end of the fp64 CPU oracle (oracle/skim_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by the cpu_baseline leg of bench.py.  The product package never imports it.
The oracle and the HIP library share no code; this module only marshals numpy
arrays into the C functions and compiles the C file with gcc when needed.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "skim_oracle.c")
_LIB = os.path.join(_HERE, "libskim_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, no FP contraction, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-std=c11", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-fPIC",
               "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_f32_to_f16.restype = C.c_uint16
        _lib.oracle_f32_to_f16.argtypes = [C.c_float]
        _lib.oracle_f16_to_f32.restype = C.c_float
        _lib.oracle_f16_to_f32.argtypes = [C.c_uint16]
        _lib.oracle_pack.restype = C.c_int64
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _p(a, ct=C.c_void_p):
    return None if a is None else a.ctypes.data_as(ct)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with status {rc}")


def scale_row(w, s, alpha):
    w, s, alpha = _f32(w), _f32(s), _f32(alpha)
    m = w.shape[0]
    wt = np.empty(m, np.float32)
    st = np.empty(m, np.float32)
    lib().oracle_scale_row(_p(w), _p(s), _p(alpha), C.c_int64(m), _p(wt), _p(st))
    return wt, st


def quantile_init(w, s, K):
    w, s = _f32(w), _f32(s)
    m = w.shape[0]
    c0 = np.empty(K, np.float64)
    ranks = np.empty(K, np.int64)
    _check(lib().oracle_quantile_init(_p(w), _p(s), C.c_int64(m), C.c_int(K), _p(c0), _p(ranks)),
           "quantile_init")
    return c0, ranks


def cluster_row(w, s, K, T=30, count_near=False):
    """One row.  Returns dict(labels, centroids, upper, err, J, near)."""
    w, s = _f32(w), _f32(s)
    m = w.shape[0]
    labels = np.empty(m, np.uint8)
    cent = np.empty(K, np.float64)
    upper = np.empty(K, np.float64)
    err = C.c_double(0)
    J = np.empty(T, np.float64)
    near = np.zeros(2, np.int64)
    _check(lib().oracle_cluster_row(_p(w), _p(s), C.c_int64(m), C.c_int(K), C.c_int(T), _p(labels),
                                    _p(cent), _p(upper), C.byref(err), _p(J),
                                    _p(near) if count_near else None), "cluster_row")
    return dict(labels=labels, centroids=cent, upper=upper, err=err.value, J=J, near=near)


def error_table(W, S, alpha=None, bmin=1, bmax=4, T=30, count_near=False):
    """Returns dict(E n x nb, centroids_all n x sum 2^b, upper_all, near[2], near_rows n, near_rb n x nb):
    near_rb[i, b] counts the decisions of row i at bit width b whose margin was below 1e-9."""
    W, S, alpha = _f32(W), _f32(S), _f32(alpha)
    n, m = W.shape
    nb = bmax - bmin + 1
    stride = sum(1 << b for b in range(bmin, bmax + 1))
    E = np.empty((n, nb), np.float64)
    ca = np.empty((n, stride), np.float64)
    ua = np.empty((n, stride), np.float64)
    near = np.zeros(2, np.int64)
    near_rows = np.zeros(n, np.int64) if count_near else None
    near_rb = np.zeros((n, nb), np.int64) if count_near else None
    _check(lib().oracle_error_table(_p(W), _p(S), _p(alpha), C.c_int64(n), C.c_int64(m),
                                    C.c_int64(m), C.c_int(bmin), C.c_int(bmax), C.c_int(T), _p(E),
                                    _p(ca), _p(ua), _p(near) if count_near else None, _p(near_rows),
                                    _p(near_rb)), "error_table")
    return dict(E=E, centroids_all=ca, upper_all=ua, near=near, near_rows=near_rows, near_rb=near_rb)


def cluster_rows(W, S, bits, alpha=None, T=30, count_near=False, want_labels=True):
    W, S, alpha = _f32(W), _f32(S), _f32(alpha)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    n, m = W.shape
    labels = np.empty((n, m), np.uint8) if want_labels else None
    cent = np.empty((n, 16), np.float64)
    upper = np.empty((n, 16), np.float64)
    err = np.empty(n, np.float64)
    near_rows = np.zeros(n, np.int64) if count_near else None
    _check(lib().oracle_cluster_rows(_p(W), _p(S), _p(alpha), C.c_int64(n), C.c_int64(m),
                                     C.c_int64(m), _p(bits), C.c_int(T), _p(labels), _p(cent),
                                     _p(upper), _p(err), _p(near_rows)), "cluster_rows")
    return dict(labels=labels, centroids=cent, upper=upper, err=err, near_rows=near_rows)


def greedy(E, avg_bits, bmin=1, bmax=4, cost=None, count_near=False):
    E = np.ascontiguousarray(E, dtype=np.float64)
    n = E.shape[0]
    assert E.shape[1] == bmax - bmin + 1
    cost_a = None if cost is None else np.ascontiguousarray(cost, dtype=np.int64)
    bits = np.empty(n, np.uint8)
    spent = C.c_int64(0)
    budget = C.c_int64(0)
    near = np.zeros(1, np.int64)
    rc = lib().oracle_greedy(_p(E), _p(cost_a), C.c_int64(n), C.c_int(bmin), C.c_int(bmax),
                             C.c_double(avg_bits), _p(bits), C.byref(spent), C.byref(budget),
                             _p(near) if count_near else None)
    if rc == -3:
        raise ValueError("budget outside [n*bmin, n*bmax]")
    _check(rc, "greedy")
    return dict(bits=bits, spent=spent.value, budget=budget.value, near=int(near[0]))


def dp_allocate(E, avg_bits, bmin=1, bmax=4):
    """Exact solution of the bit allocation problem that Alg. 1 approximates (the knapsack form stated with
    the mixed-precision problem, unit cost per row and bit): the bits b_i in [bmin, bmax] that minimise
    sum_i E[i, b_i] subject to sum_i b_i <= floor(avg_bits * n + 1e-9).

    Dynamic programme over the rows in index order: f_i[x] = least error of rows 0..i-1 when they hold
    exactly x bits above bmin in total; f_{i+1}[x] = min_d f_i[x - d] + E[i, bmin + d], where equal sums keep
    the smaller d; the answer is the smallest x that attains min_x f_n[x], traced back through the choices.
    Returns dict(bits, total, spent, budget)."""
    E = np.ascontiguousarray(E, dtype=np.float64)
    n, nb = E.shape
    assert nb == bmax - bmin + 1
    budget = int(np.floor(avg_bits * n + 1e-9))
    if budget < n * bmin or budget > n * bmax:
        raise ValueError("budget outside [n*bmin, n*bmax]")
    X = budget - n * bmin
    f = np.full(X + 1, np.inf)
    f[0] = 0.0
    choice = np.zeros((n, X + 1), np.uint8)
    for i in range(n):
        best = np.full(X + 1, np.inf)
        for d in range(nb):
            cand = np.full(X + 1, np.inf)
            cand[d:] = f[:X + 1 - d] + E[i, d]
            take = cand < best
            best[take] = cand[take]
            choice[i, take] = d
        f = best
    x = int(np.argmin(f))
    total = float(f[x])
    bits = np.empty(n, np.uint8)
    spent = n * bmin + x
    for i in range(n - 1, -1, -1):
        d = int(choice[i, x])
        bits[i] = bmin + d
        x -= d
    assert x == 0
    return dict(bits=bits, total=total, spent=spent, budget=budget)


def kmeans_optimal_row(w, s, Ks=(2, 4, 8, 16)):
    """Least weighted squared error sum_j s_j (w_j - c_{l_j})^2 of one row over ALL assignments to at most K
    clusters, for each K in Ks: the floor under what Lloyd's iterations from any start can reach.

    In one dimension an optimal assignment cuts the values, sorted, into intervals, and the best centroid of an
    interval is its weighted mean, so with the elements in the order (w, s) and prefix sums A = sum s,
    B = sum s w, C = sum s w^2:   cost(i, j) = (C_j - C_i) - (B_j - B_i)^2 / (A_j - A_i)   (elements i..j-1;
    0 when the interval holds no mass; rounding below 0 is clipped),   D_1[j] = cost(0, j),
    D_k[j] = min_{0 <= i <= j} D_{k-1}[i] + cost(i, j).   All-zero weights count as unit weights, as in the
    clustering itself.  Returns float64[len(Ks)] of D_K[m]."""
    w = np.asarray(w, np.float32).astype(np.float64)
    s = np.asarray(s, np.float32).astype(np.float64)
    m = len(w)
    if not np.any(s > 0):
        s = np.ones(m)
    order = np.lexsort((s, w))
    w, s = w[order], s[order]
    A = np.concatenate(([0.0], np.cumsum(s)))
    B = np.concatenate(([0.0], np.cumsum(s * w)))
    Cc = np.concatenate(([0.0], np.cumsum(s * w * w)))

    def cost_to(j):  # cost(i, j) for i = 0..j
        dA, dB, dC = A[j] - A[:j + 1], B[j] - B[:j + 1], Cc[j] - Cc[:j + 1]
        with np.errstate(divide="ignore", invalid="ignore"):
            c = np.where(dA > 0, dC - dB * dB / dA, 0.0)
        return np.maximum(c, 0.0)

    D = np.array([cost_to(j)[0] for j in range(m + 1)])
    out, k = [], 1
    for K in sorted(Ks):
        while k < K:
            D = np.array([np.min(D[:j + 1] + cost_to(j)) for j in range(m + 1)])
            k += 1
        out.append(D[m])
    res = dict(zip(sorted(Ks), out))
    return np.array([res[K] for K in Ks])


def kmeans_optimal_table(W, S, alpha=None, bmin=1, bmax=4):
    """kmeans_optimal_row for every row (of the scaled inputs when alpha is given) and K = 2^b, b = bmin..bmax."""
    W, S = _f32(W), _f32(S)
    out = np.empty((W.shape[0], bmax - bmin + 1))
    for i in range(W.shape[0]):
        w, s = (W[i], S[i]) if alpha is None else scale_row(W[i], S[i], alpha)
        out[i] = kmeans_optimal_row(w, s, tuple(1 << b for b in range(bmin, bmax + 1)))
    return out


def words_per_row(m, b):
    return (m * b + 31) // 32


def pack(W, bits, labels, centroids, alpha=None, want_dW=False):
    W, alpha = _f32(W), _f32(alpha)
    n, m = W.shape
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    labels = np.ascontiguousarray(labels, dtype=np.uint8)
    centroids = np.ascontiguousarray(centroids, dtype=np.float64)
    assert centroids.shape == (n, 16) and labels.shape == (n, m)
    nwords = int(sum(words_per_row(m, int(b)) for b in bits))
    ncb = int(sum(1 << int(b) for b in bits))
    codes = np.zeros(nwords, np.uint32)
    gwo = np.zeros(6, np.int64)
    perm = np.empty(n, np.int32)
    cbs = np.zeros(ncb, np.uint16)
    dW = np.empty((n, m), np.float32) if want_dW else None
    rc = lib().oracle_pack(_p(W), _p(alpha), C.c_int64(n), C.c_int64(m), C.c_int64(m), _p(bits),
                           _p(labels), _p(centroids), _p(codes), _p(gwo), _p(perm), _p(cbs), _p(dW))
    if rc < 0:
        raise RuntimeError(f"oracle pack failed with status {rc}")
    assert rc == nwords
    return dict(codes=codes, group_word_offset=gwo, row_perm=perm, codebooks=cbs, dW=dW)


def unpack(codes, group_word_offset, row_perm, codebooks, m, alpha=None):
    """Dense matrix of a packed model (layout of Sec. 4.2 / App. D.2 as `pack` writes it): rows by (bits, row),
    a b-bit row = ceil(m*b/32) little-endian uint32 words, column j at bit j*b; codebooks binary16, 2^b per row.
    Wq[i][j] = fl32(alpha_j * f32(codebook_i[code_ij])).  Rows the model does not hold stay NaN."""
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    gwo = np.asarray(group_word_offset, dtype=np.int64)
    perm = np.asarray(row_perm, dtype=np.int64)
    cbs = np.ascontiguousarray(codebooks, dtype=np.uint16).view(np.float16).astype(np.float32)
    n = len(perm)
    a = None if alpha is None else np.ascontiguousarray(alpha, dtype=np.float32)
    Wq = np.full((n, m), np.nan, np.float32)
    p = 0
    cb = 0
    j = np.arange(m, dtype=np.int64)
    for b in (1, 2, 3, 4):
        wpr = (m * b + 31) // 32
        rows = int((gwo[b + 1] - gwo[b]) // wpr)
        bit = j * b
        wi, sh = bit >> 5, (bit & 31).astype(np.uint64)
        for r in range(rows):
            w = codes[gwo[b] + r * wpr: gwo[b] + (r + 1) * wpr].astype(np.uint64)
            w = np.concatenate([w, np.zeros(1, np.uint64)])
            two = w[wi] | (w[wi + 1] << np.uint64(32))          # the 64 bits starting at the word of bit j*b
            code = ((two >> sh) & np.uint64((1 << b) - 1)).astype(np.int64)
            q = cbs[cb + code]
            Wq[perm[p]] = q if a is None else (a * q).astype(np.float32)
            p += 1
            cb += 1 << b
    return Wq


def dequant_matvec(codes, group_word_offset, row_perm, codebooks, m, x, alpha=None):
    """y = Wq x in float64 with Wq = unpack(...) (float32 weights, float32 x, products and sums float64)."""
    Wq = unpack(codes, group_word_offset, row_perm, codebooks, m, alpha)
    return Wq.astype(np.float64) @ np.ascontiguousarray(x, dtype=np.float32).astype(np.float64)


def f32_to_f16(x):
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    f = lib().oracle_f32_to_f16
    return np.array([f(float(v)) for v in x], dtype=np.uint16)


def f16_to_f32(h):
    h = np.ascontiguousarray(h, dtype=np.uint16).ravel()
    f = lib().oracle_f16_to_f32
    return np.array([f(int(v)) for v in h], dtype=np.float32)


def centroids_from_labels(W, S, labels, alpha=None):
    W, S, alpha = _f32(W), _f32(S), _f32(alpha)
    n, m = W.shape
    labels = np.ascontiguousarray(labels, dtype=np.uint8)
    c = np.empty((n, 16), np.float64)
    D = np.empty((n, 16), np.float64)
    _check(lib().oracle_centroids_from_labels(_p(W), _p(S), _p(alpha), C.c_int64(n), C.c_int64(m),
                                              C.c_int64(m), _p(labels), _p(c), _p(D)),
           "centroids_from_labels")
    return c, D


def layer_loss(W, H, labels, c, alpha=None, want_P=False):
    W, alpha, H = _f32(W), _f32(alpha), _f32(H)
    n, m = W.shape
    labels = np.ascontiguousarray(labels, dtype=np.uint8)
    c = np.ascontiguousarray(c, dtype=np.float64)
    loss = C.c_double(0)
    row_loss = np.empty(n, np.float64)
    P = np.empty((n, m), np.float64) if want_P else None
    _check(lib().oracle_layer_loss(_p(W), _p(alpha), _p(H), C.c_int64(n), C.c_int64(m),
                                   C.c_int64(m), _p(labels), _p(c), C.byref(loss), _p(row_loss),
                                   _p(P)), "layer_loss")
    return dict(loss=loss.value, row_loss=row_loss, P=P)


def error_table_lfull(W, S, H, alpha=None, bmin=1, bmax=4, iters=30, count_near=False):
    """Error pre-recording with the layer-wise error (Alg. 3, pre-recording loop, Err(.) in its L-full form):
    for each b the rows are clustered (K = 2^b), and E[i][b-bmin] = dW_i H dW_i^T with
    dW_i = w_i - alpha * replace(c, L)_i for the labels L and centroids c the clustering returned."""
    W = _f32(W)
    n, m = W.shape
    nb = bmax - bmin + 1
    E = np.empty((n, nb), np.float64)
    near_rows = np.zeros(n, np.int64)
    for b in range(bmin, bmax + 1):
        cr = cluster_rows(W, S, np.full(n, b, np.uint8), alpha=alpha, T=iters, count_near=count_near)
        E[:, b - bmin] = layer_loss(W, H, cr["labels"], cr["centroids"], alpha)["row_loss"]
        if count_near:
            near_rows += cr["near_rows"]
    return dict(E=E, near_rows=near_rows)


def scale_grad(W, S, H, labels, alpha=None):
    W, S, alpha, H = _f32(W), _f32(S), _f32(alpha), _f32(H)
    n, m = W.shape
    labels = np.ascontiguousarray(labels, dtype=np.uint8)
    loss = C.c_double(0)
    grad = np.empty(m, np.float64)
    c = np.empty((n, 16), np.float64)
    _check(lib().oracle_scale_grad(_p(W), _p(S), _p(alpha), _p(H), C.c_int64(n), C.c_int64(m),
                                   C.c_int64(m), _p(labels), C.byref(loss), _p(grad), _p(c)),
           "scale_grad")
    return dict(loss=loss.value, grad=grad, centroids=c)


ADAM_DEFAULTS = dict(lr0=0.01, beta1=0.9, beta2=0.999, eps=1e-8, decay=0.5, decay_every=40)


def adam_step(alpha, m1, m2, grad, t, **opts):
    """Updates copies of (alpha, m1, m2); returns them."""
    o = dict(ADAM_DEFAULTS)
    o.update(opts)
    alpha = np.array(alpha, dtype=np.float32, copy=True)
    m1 = np.array(m1, dtype=np.float32, copy=True)
    m2 = np.array(m2, dtype=np.float32, copy=True)
    grad = np.ascontiguousarray(grad, dtype=np.float64)
    _check(lib().oracle_adam_step(_p(alpha), _p(m1), _p(m2), _p(grad), C.c_int64(alpha.shape[0]),
                                  C.c_int64(t), C.c_double(o["lr0"]), C.c_double(o["beta1"]),
                                  C.c_double(o["beta2"]), C.c_double(o["eps"]),
                                  C.c_double(o["decay"]), C.c_int64(o["decay_every"])), "adam_step")
    return alpha, m1, m2


def hessian_from_activations(X):
    """Layer-wise Hessian proxy of Sec. 3.4 from N activation vectors (rows of X, values exactly representable
    in bfloat16): H = X^T X / N in float64, returned as float32."""
    X = np.ascontiguousarray(X, dtype=np.float32).astype(np.float64)
    return ((X.T @ X) / X.shape[0]).astype(np.float32)


def train_scale(W, S, H, bits, alpha, steps=120, outer=1, t0=1, T=30, **opts):
    """Alg. 2 as a whole: `outer` rounds of {labels = K-means of W * alpha^-1 at bits; `steps` Adam steps on
    alpha with the labels fixed}; then c = calc_centroids(W * alpha^-1, L) at the final alpha.  alpha and the
    Adam moments are float32 vectors (as in adam_step); gradients and losses are float64."""
    W, S, H = _f32(W), _f32(S), _f32(H)
    n, m = W.shape
    alpha = np.ascontiguousarray(alpha, dtype=np.float32).copy()
    m1 = np.zeros(m, np.float32)
    m2 = np.zeros(m, np.float32)
    trace = []
    t = t0
    labels = None
    for _ in range(outer):
        labels = cluster_rows(W, S, bits, alpha=alpha, T=T)["labels"]
        for _k in range(steps):
            g = scale_grad(W, S, H, labels, alpha)
            trace.append(g["loss"])
            alpha, m1, m2 = adam_step(alpha, m1, m2, g["grad"], t, **opts)
            t += 1
    c, _ = centroids_from_labels(W, S, labels, alpha)
    trace.append(layer_loss(W, H, labels, c, alpha)["loss"])
    return dict(alpha=alpha, labels=labels, centroids=c, loss_trace=np.array(trace))

