"""Shared comparison helpers of the GPU parity tests.

A decision whose oracle margin is below 1e-9 may legitimately fall the other way on the GPU (the two
sides add in different orders).  The oracle counts such decisions per (row, bit width); only those
entries are excused from the exact comparison.  An excused entry is not waved through: labels are
rebuilt from the GPU's own thresholds and the oracle's centroid and objective functions must
reproduce the GPU's centroids and error from them (valid whichever way the tie fell), and the number
of excused entries that really differ from the oracle is counted and reported.
"""
import numpy as np

import oracle

RTOL = 1e-5


def scaled_row(W, S, alpha, i):
    """The float32 values the clustering of row i consumes (unit weights for a row without mass)."""
    if alpha is None:
        wt, st = W[i], S[i]
    else:
        wt, st = oracle.scale_row(W[i], S[i], alpha)
    if not np.any(st > 0):
        st = np.ones_like(st)
    return np.ascontiguousarray(wt, np.float32), np.ascontiguousarray(st, np.float32)


def labels_from_upper(wt, upper):
    """Cluster of every value given each cluster's largest member (-inf: empty): the cluster with the
    smallest bound >= value.  Returns None when some value lies above every bound."""
    order = np.argsort(upper, kind="stable")
    us = upper[order]
    pos = np.searchsorted(us, wt.astype(np.float64), side="left")
    if pos.max() >= len(us):
        return None
    return order[pos].astype(np.uint8)


def entry_self_check(wt, st, c_gpu, u_gpu, e_gpu, rtol=RTOL):
    """Self-consistency of one (row, bit width) result through the oracle's functions.  Returns an error
    string or None."""
    u = np.asarray(u_gpu, np.float64)
    fin = np.isfinite(u)
    if not fin.any():
        return "no cluster has a member"
    if not np.isin(u[fin], wt.astype(np.float64)).all():
        return "a threshold is not a value of the row"
    if len(np.unique(u[fin])) != int(fin.sum()):
        return "two clusters share a threshold"
    lab = labels_from_upper(wt, u)
    if lab is None:
        return "a value lies above every threshold"
    c, D = oracle.centroids_from_labels(wt[None], st[None], lab[None])
    c, D = c[0, :len(u)], D[0, :len(u)]
    wscale = float(np.abs(wt).max())
    live = D > 0
    bad = np.abs(c_gpu[live] - c[live]) > rtol * np.abs(c[live]) + 1e-12 * wscale
    if bad.any():
        return f"centroids are not the weighted means of their clusters (max diff {np.abs(c_gpu[live] - c[live]).max():.3e})"
    w64, s64 = wt.astype(np.float64), st.astype(np.float64)
    J = float(np.sum(s64 * (w64 - np.asarray(c_gpu, np.float64)[lab]) ** 2))
    scale = float(np.sum(s64 * w64 * w64))
    if abs(J - e_gpu) > rtol * J + 1e-13 * scale:
        return f"error {e_gpu!r} is not the objective of the labels {J!r}"
    return None


def compare_table(W, S, alpha, ref, E, ca, ua, bmin=1, bmax=4, rtol=RTOL):
    """Entry-by-entry comparison of an error table with the oracle's (ref from oracle.error_table with
    count_near=True).  Clean entries: thresholds bit-exact, errors and centroids within rtol.  Excused
    entries: entry_self_check.  Returns dict(excused, differ, max_gap, max_rel)."""
    n, m = W.shape
    near = ref["near_rb"]
    clean = near == 0
    ua = np.asarray(ua, np.float64)
    row_scale = np.empty(n)
    wscale = np.empty(n)
    for i in range(n):
        if alpha is None and np.any(S[i] > 0):
            w64 = W[i].astype(np.float64)
            row_scale[i] = float(np.sum(S[i].astype(np.float64) * w64 * w64))
            wscale[i] = float(np.abs(W[i]).max())
        else:
            wt, st = scaled_row(W, S, alpha, i)
            w64 = wt.astype(np.float64)
            row_scale[i] = float(np.sum(st.astype(np.float64) * w64 * w64))
            wscale[i] = float(np.abs(wt).max())
    assert np.isfinite(E).all() and (E >= 0).all()
    max_rel = 0.0
    off = 0
    differ = 0
    max_gap = 0.0
    for bi, b in enumerate(range(bmin, bmax + 1)):
        K = 1 << b
        sl = slice(off, off + K)
        off += K
        cl = clean[:, bi]
        bad_u = (ua[cl][:, sl] != ref["upper_all"][cl][:, sl]).any(1)
        assert not bad_u.any(), (f"b={b}: thresholds differ in {int(bad_u.sum())} clean rows, first "
                                 f"{np.flatnonzero(cl)[np.flatnonzero(bad_u)[:5]].tolist()}")
        dE = np.abs(E[cl, bi] - ref["E"][cl, bi])
        okE = (dE <= rtol * ref["E"][cl, bi]) | (dE <= 1e-13 * row_scale[cl])
        assert okE.all(), f"b={b}: E differs, max rel {np.max(dE / np.maximum(ref['E'][cl, bi], 1e-300)):.3e}"
        if cl.any():
            nz = ref["E"][cl, bi] > 1e-13 * row_scale[cl]
            if nz.any():
                max_rel = max(max_rel, float(np.max(dE[nz] / ref["E"][cl, bi][nz])))
        cd = np.abs(ca[cl][:, sl] - ref["centroids_all"][cl][:, sl])
        okc = cd <= rtol * np.abs(ref["centroids_all"][cl][:, sl]) + 1e-12 * wscale[cl, None]
        assert okc.all(), f"b={b}: centroids differ at rows {np.flatnonzero(cl)[np.argwhere(~okc)[:5, 0]].tolist()}, max {cd.max():.3e}"
        for i in np.flatnonzero(~cl):
            wt, st = scaled_row(W, S, alpha, i)
            msg = entry_self_check(wt, st, ca[i, sl], ua[i, sl], float(E[i, bi]), rtol)
            assert msg is None, f"row {i}, b={b} (excused from the exact comparison): {msg}"
            if (ua[i, sl] != ref["upper_all"][i, sl]).any():
                differ += 1
                if ref["E"][i, bi] > 0:
                    max_gap = max(max_gap, abs(float(E[i, bi]) - ref["E"][i, bi]) / ref["E"][i, bi])
    excused = int((~clean).sum())
    assert differ <= excused
    return dict(excused=excused, differ=differ, max_gap=max_gap, max_rel=max_rel, clean=clean)


def check_rows_self_consistent(W, S, alpha, bits, labels, centroids, upper, err, rows=None, rtol=RTOL):
    """cluster_rows outputs of the given rows (default all): labels are what the thresholds say, centroids
    the weighted means of the labels, err the objective (through the oracle's functions)."""
    n = W.shape[0]
    rows = range(n) if rows is None else rows
    for i in rows:
        K = 1 << int(bits[i])
        wt, st = scaled_row(W, S, alpha, i)
        lab = labels_from_upper(wt, np.asarray(upper[i, :K], np.float64))
        assert lab is not None and np.array_equal(lab, labels[i]), f"row {i}: labels do not follow from the thresholds"
        msg = entry_self_check(wt, st, centroids[i, :K], upper[i, :K], float(err[i]), rtol)
        assert msg is None, f"row {i}: {msg}"
