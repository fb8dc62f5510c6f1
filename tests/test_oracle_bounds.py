"""Pins for the oracle's exact bounds (no GPU): the knapsack optimum of the bit allocation problem and the
least error any assignment of a row to K clusters can have."""
import itertools

import numpy as np
import pytest

import oracle


# ---------------------------------------------------------------- exact allocation
def brute_force_at_most(E, budget, bmin, bmax):
    best, best_bits = np.inf, None
    for bits in itertools.product(range(bmin, bmax + 1), repeat=E.shape[0]):   # lexicographic order
        if sum(bits) > budget:
            continue
        tot = 0.0
        for i, b in enumerate(bits):      # same order of additions as the recurrence
            tot = tot + E[i, b - bmin]
        if tot < best:
            best, best_bits = tot, bits
    return best, best_bits


@pytest.mark.parametrize("seed", range(8))
def test_dp_allocation_is_the_exhaustive_optimum(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 7))
    E = rng.uniform(0, 10, (n, 4))            # gains of either sign, in any order
    for avg in (1.0, 1.5, 2.0, 2.6, 3.2, 4.0):
        r = oracle.dp_allocate(E, avg)
        B = int(np.floor(n * avg + 1e-9))
        opt, _ = brute_force_at_most(E, B, 1, 4)
        assert r["total"] == pytest.approx(opt, rel=1e-14)
        assert r["budget"] == B and r["spent"] == int(r["bits"].sum()) <= B
        assert sum(E[i, b - 1] for i, b in enumerate(r["bits"])) == pytest.approx(r["total"], rel=1e-14)


@pytest.mark.parametrize("seed", range(6))
def test_dp_equals_greedy_for_diminishing_returns_and_never_loses(seed):
    """Greedy is optimal when every row's reductions are positive and shrink with bits (marginal analysis);
    on any table it can only be worse or equal."""
    rng = np.random.default_rng(100 + seed)
    n = 40
    gains = np.sort(rng.uniform(0.1, 5.0, (n, 3)), axis=1)[:, ::-1]
    E = np.empty((n, 4))
    E[:, 0] = rng.uniform(20, 30, n)
    for b in range(3):
        E[:, b + 1] = E[:, b] - gains[:, b]
    for avg in (1.5, 2.25, 3.2):
        g = oracle.greedy(E, avg)
        r = oracle.dp_allocate(E, avg)
        gt = sum(E[i, b - 1] for i, b in enumerate(g["bits"]))
        assert r["total"] == pytest.approx(gt, rel=1e-13)
        assert r["spent"] == r["budget"]
    E2 = rng.uniform(0, 10, (n, 4))
    for avg in (1.5, 2.25, 3.2):
        g = oracle.greedy(E2, avg)
        gt = sum(E2[i, b - 1] for i, b in enumerate(g["bits"]))
        assert oracle.dp_allocate(E2, avg)["total"] <= gt + 1e-12


def test_dp_leaves_bits_unspent_when_more_bits_hurt_and_ties_take_fewer_bits():
    E = np.array([[5.0, 6.0, 7.0, 8.0],     # every extra bit makes this row worse
                  [5.0, 4.0, 3.0, 2.0],
                  [1.0, 1.0, 1.0, 1.0]])    # nothing to gain: equal sums keep the fewer bits
    r = oracle.dp_allocate(E, 4.0)
    assert np.array_equal(r["bits"], [1, 4, 1]) and r["spent"] == 6 and r["budget"] == 12 and r["total"] == 8.0
    r = oracle.dp_allocate(E, 5 / 3 + 1e-12)      # two spare bits
    assert np.array_equal(r["bits"], [1, 3, 1]) and r["total"] == 9.0
    with pytest.raises(ValueError):
        oracle.dp_allocate(E, 0.9)
    with pytest.raises(ValueError):
        oracle.dp_allocate(E, 4.4)


def test_jump_in_returns_where_greedy_is_beaten():
    """A row whose big reduction sits behind a small one: greedy looks one bit ahead and misses it."""
    E = np.array([[10.0, 9.9, 0.0],
                  [10.0, 8.0, 7.0]])
    g = oracle.greedy(E, 2.0, bmin=1, bmax=3)          # 2 spare bits
    assert np.array_equal(g["bits"], [1, 3])           # 2.0 then 1.0: total 17
    r = oracle.dp_allocate(E, 2.0, bmin=1, bmax=3)
    assert np.array_equal(r["bits"], [3, 1]) and r["total"] == 10.0


def test_floor_initialised_allocation():
    """The variant for non-integer targets that starts every row at floor(target) bits (appendix on the OPT
    models): Alg. 1 on the columns floor..bmax.  Then every row has floor or floor + 1 bits when the
    reductions are positive, and the rows with the largest one-bit reductions are the ones upgraded."""
    rng = np.random.default_rng(3)
    n = 500
    E = np.sort(rng.uniform(0, 10, (n, 4)), axis=1)[:, ::-1].copy()
    target = 3.2
    fl = int(np.floor(target))
    g = oracle.greedy(E[:, fl - 1:], target, bmin=fl, bmax=4)
    assert set(np.unique(g["bits"])) == {3, 4} and g["spent"] == g["budget"] == 1600
    up = np.flatnonzero(g["bits"] == 4)
    gain = E[:, 2] - E[:, 3]
    want = np.sort(np.lexsort((np.arange(n), -gain))[:100])
    assert np.array_equal(up, want)
    # at an integer target the variant has no freedom left
    g = oracle.greedy(E[:, 2:3], 3.0, bmin=3, bmax=3)
    assert np.all(g["bits"] == 3)


# ---------------------------------------------------------------- optimal 1-D clustering
def direct_error(w, s, labels, K):
    tot = 0.0
    for p in range(K):
        sel = labels == p
        mass = s[sel].sum()
        if mass > 0:
            c = (s[sel] * w[sel]).sum() / mass
            tot += (s[sel] * (w[sel] - c) ** 2).sum()
    return tot


@pytest.mark.parametrize("seed", range(6))
def test_optimal_row_against_every_assignment(seed):
    rng = np.random.default_rng(seed)
    m = 8
    w = rng.standard_normal(m).astype(np.float32)
    if seed % 2:
        w[rng.integers(0, m, 3)] = w[0]                      # repeated values
    s = rng.uniform(0.1, 2.0, m).astype(np.float32)
    if seed % 3 == 0:
        s[rng.integers(0, m, 2)] = 0                         # weightless elements
    w64, s64 = w.astype(np.float64), s.astype(np.float64)
    for K in (1, 2, 3):
        best = min(direct_error(w64, s64, np.array(lab), K) for lab in itertools.product(range(K), repeat=m))
        got = oracle.kmeans_optimal_row(w, s, (K,))[0]
        assert got == pytest.approx(best, rel=1e-9, abs=1e-13)


def test_optimal_row_closed_forms():
    # unit weights on 0..m-1: K equal runs of q consecutive integers are optimal, each with SSE q(q^2-1)/12
    for K, q in ((2, 6), (4, 5), (8, 3), (16, 4)):
        w = np.arange(K * q, dtype=np.float32)
        got = oracle.kmeans_optimal_row(w, np.ones_like(w), (K,))[0]
        assert got == pytest.approx(K * q * (q * q - 1) / 12.0, rel=1e-12)
    # K = 1 is the weighted variance times the mass
    rng = np.random.default_rng(0)
    w = rng.standard_normal(200).astype(np.float32)
    s = rng.uniform(0, 1, 200).astype(np.float32)
    w64, s64 = w.astype(np.float64), s.astype(np.float64)
    mu = (s64 * w64).sum() / s64.sum()
    assert oracle.kmeans_optimal_row(w, s, (1,))[0] == pytest.approx((s64 * (w64 - mu) ** 2).sum(), rel=1e-11)
    # no more distinct values than clusters: nothing is lost; all-zero weights count as ones
    w = np.repeat(np.float32([-1.5, 0.25, 3.0, 7.0]), 5)
    assert oracle.kmeans_optimal_row(w, np.ones_like(w), (4, 8)) == pytest.approx([0, 0], abs=1e-12)
    assert oracle.kmeans_optimal_row(w, np.zeros_like(w), (2,))[0] == \
        pytest.approx(oracle.kmeans_optimal_row(w, np.ones_like(w), (2,))[0], rel=1e-14)
    assert oracle.kmeans_optimal_row(w, np.ones_like(w), (2,))[0] > 1.0


@pytest.mark.parametrize("seed", range(4))
def test_optimal_row_bounds_lloyd_and_ignores_weightless_elements(seed):
    rng = np.random.default_rng(10 + seed)
    m = 300
    w = (rng.standard_t(4, m) * 0.02).astype(np.float32)
    s = (rng.lognormal(0, 1.5, m) * 1e-4).astype(np.float32)
    opt = oracle.kmeans_optimal_row(w, s)
    assert np.all(np.diff(opt) <= 0)
    for K, o in zip((2, 4, 8, 16), opt):
        lloyd = oracle.cluster_row(w, s, K)["err"]
        assert o <= lloyd * (1 + 1e-9)
    w2 = np.concatenate([w, rng.standard_normal(40).astype(np.float32)])
    s2 = np.concatenate([s, np.zeros(40, np.float32)])
    assert oracle.kmeans_optimal_row(w2, s2) == pytest.approx(opt, rel=1e-9)
