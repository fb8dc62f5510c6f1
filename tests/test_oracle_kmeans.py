"""Pins for the K-means part of the CPU oracle (no GPU).

The paper prints no worked example, so the oracle is pinned to mathematics:
exact 1-D K-means by dynamic programming, numpy's weighted inverted-CDF
quantile, closed forms, exact power-of-two symmetries, a hand-worked case.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
import skim_synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_fixture(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split("=")
            out[k.strip()] = np.array([float(x) for x in v.split()])
    return out


def exact_kmeans_dp(w, s, K):
    """Optimal weighted 1-D K-means cost by dynamic programming over the sorted
    row (optimal clusters are contiguous in value).  O(K m^2), exact up to fp64."""
    order = np.argsort(w, kind="stable")
    w = np.asarray(w, np.float64)[order]
    s = np.asarray(s, np.float64)[order]
    m = len(w)
    P0 = np.concatenate([[0.0], np.cumsum(s)])
    P1 = np.concatenate([[0.0], np.cumsum(s * w)])
    P2 = np.concatenate([[0.0], np.cumsum(s * w * w)])

    def cost(a, b):  # elements a..b-1
        d = P0[b] - P0[a]
        if d <= 0:
            return 0.0
        n1 = P1[b] - P1[a]
        return max(0.0, (P2[b] - P2[a]) - n1 * n1 / d)

    INF = float("inf")
    best = [[INF] * (m + 1) for _ in range(K + 1)]
    best[0][0] = 0.0
    for k in range(1, K + 1):
        for b in range(k, m + 1):
            v = INF
            for a in range(k - 1, b):
                if best[k - 1][a] < INF:
                    v = min(v, best[k - 1][a] + cost(a, b))
            best[k][b] = v
    return best[K][m]


def objective(w, s, labels, c):
    w = np.asarray(w, np.float64)
    s = np.asarray(s, np.float64)
    return float(np.sum(s * (w - c[labels]) ** 2))


def test_hand_worked_example():
    fx = read_fixture("kmeans_hand_worked.txt")
    w = fx["w"].astype(np.float32)
    s = fx["s"].astype(np.float32)
    c0, ranks = oracle.quantile_init(w, s, 2)
    assert np.array_equal(c0, fx["init"])
    r = oracle.cluster_row(w, s, 2, T=30)
    assert np.array_equal(r["labels"], fx["labels"].astype(np.uint8))
    assert np.array_equal(r["centroids"], fx["centroids"])
    assert r["err"] == fx["err"][0]
    assert exact_kmeans_dp(w, s, 2) == pytest.approx(fx["optimum"][0], rel=1e-14)
    assert np.array_equal(r["upper"], [-2.0, 7.0])


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("K", [2, 4, 8])
def test_lloyd_never_beats_exact_dp(seed, K):
    rng = np.random.default_rng(seed)
    m = int(rng.integers(K, 49))
    w = rng.standard_normal(m).astype(np.float32)
    s = (rng.standard_t(3, m) ** 2).astype(np.float32)
    r = oracle.cluster_row(w, s, K)
    opt = exact_kmeans_dp(w, s, K)
    assert r["err"] >= opt * (1 - 1e-12) - 1e-300
    # the reported error is the objective of the reported labels/centroids
    assert r["err"] == pytest.approx(objective(w, s, r["labels"], r["centroids"]), rel=1e-12)


@pytest.mark.parametrize("K", [2, 4, 8, 16])
def test_well_separated_clusters_reach_the_optimum(K):
    rng = np.random.default_rng(K)
    per = 4
    centers = np.arange(K) * 10.0
    w = (centers[:, None] + rng.uniform(-0.5, 0.5, (K, per))).ravel().astype(np.float32)
    s = rng.uniform(0.5, 1.5, K * per).astype(np.float32)
    perm = rng.permutation(K * per)
    w, s = w[perm], s[perm]
    r = oracle.cluster_row(w, s, K)
    assert r["err"] == pytest.approx(exact_kmeans_dp(w, s, K), rel=1e-10)
    # labels = index of the blob, in ascending order of value
    assert np.array_equal(r["labels"], np.round(w / 10.0).astype(np.uint8))


@pytest.mark.parametrize("seed", range(6))
def test_objective_non_increasing_and_centroids_are_weighted_means(seed):
    W, S = skim_synth.make_ws_small(seed, 1, 300 + 37 * seed)
    w, s = W[0], S[0]
    for K in (2, 4, 8, 16):
        r = oracle.cluster_row(w, s, K, T=30)
        J = r["J"]
        assert np.all(np.diff(J) <= 1e-12 * J[:-1])
        assert J[-1] == r["err"]
        sd, wd = s.astype(np.float64), w.astype(np.float64)
        for k in range(K):
            mem = r["labels"] == k
            D, N = sd[mem].sum(), (sd[mem] * wd[mem]).sum()
            if D > 0:
                assert r["centroids"][k] * D == pytest.approx(N, rel=1e-12, abs=1e-300)
                assert r["upper"][k] == wd[mem].max()
            if not mem.any():
                assert r["upper"][k] == -np.inf


def test_iteration_chain_matches_library_argmin():
    """Labels after T+1 iterations are numpy's nearest-centroid labels with
    respect to the centroids after T iterations (first minimum wins)."""
    W, S = skim_synth.make_ws_small(3, 1, 257)
    w, s = W[0], S[0]
    K = 8
    prev = oracle.cluster_row(w, s, K, T=1)
    c0, _ = oracle.quantile_init(w, s, K)
    lab = np.argmin(np.abs(w.astype(np.float64)[:, None] - c0[None, :]), axis=1)
    assert np.array_equal(prev["labels"], lab.astype(np.uint8))
    for T in range(2, 8):
        cur = oracle.cluster_row(w, s, K, T=T)
        lab = np.argmin(np.abs(w.astype(np.float64)[:, None] - prev["centroids"][None, :]), axis=1)
        assert np.array_equal(cur["labels"], lab.astype(np.uint8))
        prev = cur


@pytest.mark.parametrize("seed", range(5))
def test_quantile_init_matches_numpy_weighted_quantile(seed):
    rng = np.random.default_rng(100 + seed)
    m = 400
    w = rng.standard_normal(m).astype(np.float32)
    s = rng.uniform(0.5, 1.5, m).astype(np.float32)  # no dominant element -> no rank repair
    for K in (2, 4, 8, 16):
        c0, ranks = oracle.quantile_init(w, s, K)
        q = (2 * np.arange(K) + 1) / (2 * K)
        ref = np.quantile(w.astype(np.float64), q, weights=s.astype(np.float64), method="inverted_cdf")
        assert np.array_equal(c0, ref)
        assert np.all(np.diff(ranks) > 0)


def test_quantile_init_unit_weights_closed_form():
    m = 1000
    w = np.random.default_rng(5).permutation(m).astype(np.float32)  # sorted value == rank
    s = np.ones(m, np.float32)
    for K in (2, 4, 8, 16):
        c0, ranks = oracle.quantile_init(w, s, K)
        expect = np.ceil(m * (2 * np.arange(K) + 1) / (2 * K)) - 1
        assert np.array_equal(ranks, expect.astype(np.int64))
        assert np.array_equal(c0, expect)


def test_quantile_init_rank_repair_gives_distinct_elements():
    # one element carries almost all mass: every target falls on its rank
    m, K = 40, 8
    w = np.arange(m, dtype=np.float32)
    s = np.full(m, 1e-6, np.float32)
    s[10] = 1e6
    c0, ranks = oracle.quantile_init(w, s, K)
    assert np.array_equal(ranks, 10 + np.arange(K))
    # heavy element at the very end: ranks are pushed down to leave room
    s = np.full(m, 1e-6, np.float32)
    s[m - 1] = 1e6
    c0, ranks = oracle.quantile_init(w, s, K)
    assert np.array_equal(ranks, m - K + np.arange(K))


def test_order_among_equal_values_is_by_sensitivity():
    # equal w: the (w, s, index) order makes the result independent of column order
    w = np.array([1, 1, 1, 1, 2, 3, 4, 5], np.float32)
    s = np.array([4, 1, 3, 2, 1, 1, 1, 1], np.float32)
    c_a, r_a = oracle.quantile_init(w, s, 4)
    perm = np.array([3, 0, 2, 1, 7, 5, 6, 4])
    c_b, r_b = oracle.quantile_init(w[perm], s[perm], 4)
    assert np.array_equal(c_a, c_b) and np.array_equal(r_a, r_b)


def test_single_cluster_closed_form():
    W, S = skim_synth.make_ws_small(11, 1, 500)
    w, s = W[0].astype(np.float64), S[0].astype(np.float64)
    r = oracle.cluster_row(W[0], S[0], 1)
    mean = (s * w).sum() / s.sum()
    assert r["centroids"][0] == pytest.approx(mean, rel=1e-13)
    assert r["err"] == pytest.approx((s * (w - mean) ** 2).sum(), rel=1e-12)
    assert np.all(r["labels"] == 0)


def test_as_many_clusters_as_elements_gives_zero_error():
    w = np.array([0.3, -1.0, 2.5, 0.1, 7.0, -3.0, 0.2, 1.0], np.float32)
    s = np.array([1, 2, 3, 4, 5, 6, 7, 8], np.float32)
    r = oracle.cluster_row(w, s, 8)
    assert r["err"] == 0.0
    assert np.array_equal(np.sort(r["centroids"]), np.sort(w.astype(np.float64)))
    assert np.array_equal(r["labels"], np.argsort(np.argsort(w)).astype(np.uint8))


@pytest.mark.parametrize("p,q", [(3, 0), (-5, 2), (0, -7), (4, 4)])
def test_power_of_two_scaling_is_exact(p, q):
    W, S = skim_synth.make_ws_small(21, 1, 333)
    w, s = W[0], S[0]
    for K in (4, 16):
        a = oracle.cluster_row(w, s, K)
        b = oracle.cluster_row(w * np.float32(2.0 ** p), s * np.float32(2.0 ** q), K)
        assert np.array_equal(a["labels"], b["labels"])
        assert np.array_equal(a["centroids"] * 2.0 ** p, b["centroids"])
        assert a["err"] * 2.0 ** (2 * p + q) == b["err"]


def test_column_permutation_permutes_labels():
    W, S = skim_synth.make_ws_small(22, 1, 200)
    w, s = W[0], S[0]
    perm = np.random.default_rng(0).permutation(200)
    for K in (2, 8):
        a = oracle.cluster_row(w, s, K, T=5)
        b = oracle.cluster_row(w[perm], s[perm], K, T=5)
        assert np.array_equal(a["labels"][perm], b["labels"])
        # sums run in a different order: centroids agree to rounding only
        np.testing.assert_allclose(a["centroids"], b["centroids"], rtol=1e-12)


def test_zero_total_sensitivity_uses_unit_weights():
    w = np.random.default_rng(3).standard_normal(64).astype(np.float32)
    z = np.zeros(64, np.float32)
    one = np.ones(64, np.float32)
    a = oracle.cluster_row(w, z, 4)
    b = oracle.cluster_row(w, one, 4)
    assert np.array_equal(a["labels"], b["labels"])
    assert np.array_equal(a["centroids"], b["centroids"])
    assert a["err"] == b["err"]


def test_cluster_without_mass_keeps_its_centroid():
    # the two middle elements have zero sensitivity and form their own cluster
    w = np.array([0.0, 0.1, 5.0, 5.1, 10.0, 10.1], np.float32)
    s = np.array([1, 1, 0, 0, 1, 1], np.float32)
    # K = 3: ranks from targets 2/3, 2, 10/3 over running sums 1 2 2 2 3 4 -> 0, 1->., see below
    c0, ranks = oracle.quantile_init(w, s, 3)
    r = oracle.cluster_row(w, s, 3)
    # every centroid is either a weighted mean of members with mass or an initial value
    for k in range(3):
        mem = r["labels"] == k
        D = s[mem].astype(np.float64).sum()
        if D == 0:
            assert r["centroids"][k] in c0
    assert r["err"] == pytest.approx(objective(w, s, r["labels"], r["centroids"]), rel=1e-14)


def test_duplicate_start_values_lowest_index_wins():
    # duplicate values at adjacent ranks -> two equal starting centroids; the
    # first of them takes every member, the second keeps its value.
    w = np.array([1, 1, 1, 1, 1, 1, 9, 9], np.float32)
    s = np.array([1, 1, 1, 1, 1, 1, 1, 1], np.float32)
    c0, ranks = oracle.quantile_init(w, s, 4)
    assert np.array_equal(c0, [1, 1, 1, 9])
    r = oracle.cluster_row(w, s, 4)
    assert np.array_equal(r["labels"], [0, 0, 0, 0, 0, 0, 3, 3])
    assert np.array_equal(r["centroids"], [1, 1, 1, 9])
    assert r["upper"][1] == -np.inf and r["upper"][2] == -np.inf


def test_brute_force_assignment_optimum_tiny():
    """On 7 elements, K = 3: exhaustive search over all 3^7 labelings gives the
    global optimum of the objective; DP must equal it and Lloyd must not beat it."""
    rng = np.random.default_rng(9)
    w = rng.standard_normal(7).astype(np.float32)
    s = rng.uniform(0.1, 2.0, 7).astype(np.float32)
    wd, sd = w.astype(np.float64), s.astype(np.float64)
    best = np.inf
    for lab in itertools.product(range(3), repeat=7):
        lab = np.array(lab)
        J = 0.0
        for k in range(3):
            mem = lab == k
            if mem.any():
                c = (sd[mem] * wd[mem]).sum() / sd[mem].sum()
                J += (sd[mem] * (wd[mem] - c) ** 2).sum()
        best = min(best, J)
    assert exact_kmeans_dp(w, s, 3) == pytest.approx(best, rel=1e-12)
    assert oracle.cluster_row(w, s, 3)["err"] >= best * (1 - 1e-12)


def test_scaled_row_is_single_precision_division_and_products():
    W, S = skim_synth.make_ws_small(31, 1, 1000)
    al = skim_synth.make_alpha(1, 1000)
    wt, st = oracle.scale_row(W[0], S[0], al)
    assert np.array_equal(wt, W[0] / al)                      # numpy float32 ops are IEEE single
    assert np.array_equal(st, (S[0] * al) * al)
    wt1, st1 = oracle.scale_row(W[0], S[0], None)
    assert np.array_equal(wt1, W[0]) and np.array_equal(st1, S[0])


def test_error_table_rows_equal_single_row_calls_and_config0_has_no_near_ties():
    W, S = skim_synth.make_ws(0)
    tab = oracle.error_table(W, S, count_near=True)
    assert tab["near"].tolist() == [0, 0]
    E = tab["E"]
    assert E.shape == (512, 4)
    for i in (0, 17, 511):
        off = 0
        for bi, b in enumerate((1, 2, 3, 4)):
            r = oracle.cluster_row(W[i], S[i], 1 << b)
            assert r["err"] == E[i, bi]
            assert np.array_equal(r["centroids"], tab["centroids_all"][i, off:off + (1 << b)])
            assert np.array_equal(r["upper"], tab["upper_all"][i, off:off + (1 << b)])
            off += 1 << b
    # more centroids from a refined start lower the error for almost every row
    assert np.mean(E[:, 1:] <= E[:, :-1]) > 0.99


def test_cluster_rows_matches_table_blocks():
    W, S = skim_synth.make_ws(0, rows=64)
    tab = oracle.error_table(W, S)
    bits = (np.arange(64) % 4 + 1).astype(np.uint8)
    cr = oracle.cluster_rows(W, S, bits)
    offs = {1: 0, 2: 2, 3: 6, 4: 14}
    for i in range(64):
        b = int(bits[i])
        assert cr["err"][i] == tab["E"][i, b - 1]
        assert np.array_equal(cr["centroids"][i, :1 << b], tab["centroids_all"][i, offs[b]:offs[b] + (1 << b)])
        assert np.all(cr["labels"][i] < (1 << b))


def test_shape_errors():
    w = np.zeros(3, np.float32)
    with pytest.raises(RuntimeError):
        oracle.cluster_row(w, w, 4)
