"""Pins for the allocation and packing parts of the CPU oracle (no GPU)."""
import itertools
import os

import numpy as np
import pytest

import oracle
import skim_synth
from test_oracle_kmeans import read_fixture


# ---------------------------------------------------------------- allocation
def brute_force_alloc(E, budget, bmin, bmax):
    n = E.shape[0]
    best, best_bits = np.inf, None
    for bits in itertools.product(range(bmin, bmax + 1), repeat=n):
        if sum(bits) != budget:
            continue
        tot = sum(E[i, b - bmin] for i, b in enumerate(bits))
        if tot < best:
            best, best_bits = tot, bits
    return best, best_bits


def test_hand_worked_allocation():
    fx = read_fixture("alloc_hand_worked.txt")
    E = np.stack([fx["E0"], fx["E1"], fx["E2"]])
    g = oracle.greedy(E, 2.0, bmin=1, bmax=3)
    assert np.array_equal(g["bits"], fx["bits"].astype(np.uint8))
    assert g["spent"] == g["budget"] == 6
    tot = sum(E[i, b - 1] for i, b in enumerate(g["bits"]))
    assert tot == fx["total"][0]
    opt, opt_bits = brute_force_alloc(E, 6, 1, 3)
    assert opt == fx["optimum"][0] and np.array_equal(opt_bits, fx["optimum_bits"])


@pytest.mark.parametrize("seed", range(10))
def test_greedy_is_optimal_for_diminishing_returns(seed):
    """Marginal analysis: when every row's reductions shrink with bits, greedy
    reaches the exhaustive-search optimum."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(3, 8))
    gains = np.sort(rng.uniform(0.1, 5.0, (n, 3)), axis=1)[:, ::-1]  # decreasing
    E = np.empty((n, 4))
    E[:, 0] = rng.uniform(20, 30, n)
    for b in range(3):
        E[:, b + 1] = E[:, b] - gains[:, b]
    for avg in (1.5, 2.0, 2.4, 3.0, 3.7):
        g = oracle.greedy(E, avg)
        B = int(np.floor(n * avg + 1e-9))
        assert g["budget"] == B and g["spent"] == B and int(g["bits"].sum()) == B
        tot = sum(E[i, b - 1] for i, b in enumerate(g["bits"]))
        opt, _ = brute_force_alloc(E, B, 1, 4)
        assert tot == pytest.approx(opt, rel=1e-13)


@pytest.mark.parametrize("seed", range(6))
def test_greedy_budget_met_exactly_and_never_beats_optimum(seed):
    rng = np.random.default_rng(50 + seed)
    n = 7
    E = np.sort(rng.uniform(0, 10, (n, 4)), axis=1)[:, ::-1].copy()  # decreasing errors, arbitrary gains
    for avg in (1.0, 2.25, 3.2, 4.0):
        g = oracle.greedy(E, avg)
        B = int(np.floor(n * avg + 1e-9))
        assert int(g["bits"].sum()) == B == g["spent"]
        assert g["bits"].min() >= 1 and g["bits"].max() <= 4
        tot = sum(E[i, b - 1] for i, b in enumerate(g["bits"]))
        opt, _ = brute_force_alloc(E, B, 1, 4)
        assert tot >= opt - 1e-12


def test_greedy_negative_gains_taken_last_and_ties_lowest_index():
    E = np.array([[5.0, 6.0, 7.0, 8.0],    # more bits make it worse (local optimum of Lloyd)
                  [5.0, 4.0, 3.0, 2.0],
                  [5.0, 4.0, 3.0, 2.0]])
    g = oracle.greedy(E, 2.0)              # 3 upgrades
    assert np.array_equal(g["bits"], [1, 4, 1])     # equal reductions: lowest row index every time
    g = oracle.greedy(E, 10 / 3 + 1e-12)   # 7 upgrades: rows 1,2 saturate, row 0 takes one
    assert np.array_equal(g["bits"], [2, 4, 4])


def test_greedy_budget_errors_and_floor():
    E = np.zeros((10, 4))
    with pytest.raises(ValueError):
        oracle.greedy(E, 0.5)
    with pytest.raises(ValueError):
        oracle.greedy(E, 4.5)
    assert oracle.greedy(E, 2.25)["budget"] == 22     # floor(22.5)
    assert oracle.greedy(E, 3.2)["budget"] == 32      # 3.2*10 is not exact in binary; 1e-9 guard
    assert oracle.greedy(E, 2.5)["spent"] == 25


def test_greedy_with_row_costs():
    # two wide rows (cost 3) and three narrow rows (cost 1); density = reduction / cost
    E = np.array([[30.0, 0.0, 0.0, 0.0],     # reduction 30 at cost 3 -> density 10
                  [12.0, 3.0, 0.0, 0.0],     # 9 / 3 = 3
                  [8.0, 1.0, 0.5, 0.4],      # 7
                  [6.0, 1.0, 0.5, 0.4],      # 5
                  [2.0, 1.9, 1.8, 1.7]])
    cost = np.array([3, 3, 1, 1, 1])
    csum = 9
    g = oracle.greedy(E, (csum + 5) / csum, cost=cost)   # 5 spare bits
    assert g["budget"] == 14
    # order: row0 (10, 3 bits), row2 (7, 1 bit), row3 (5, 1 bit) -> 0 bits left
    assert np.array_equal(g["bits"], [2, 1, 2, 2, 1])
    assert g["spent"] == 14
    g = oracle.greedy(E, (csum + 4) / csum, cost=cost)   # 4 spare: row0, then row2; row3 still fits (1 left -> yes)
    assert g["spent"] <= g["budget"]
    left = g["budget"] - g["spent"]
    upgradable = [cost[i] for i in range(5) if g["bits"][i] < 4]
    assert all(c > left for c in upgradable) or left == 0


def test_greedy_config0_table():
    W, S = skim_synth.make_ws(0)
    E = oracle.error_table(W, S)["E"]
    g = oracle.greedy(E, 3.0, count_near=True)
    assert g["budget"] == 1536 and g["spent"] == 1536 and int(g["bits"].sum()) == 1536
    assert g["near"] == 0


# ---------------------------------------------------------------- fp16
def test_f16_conversion_matches_numpy_everywhere():
    halves = np.arange(65536, dtype=np.uint16)
    as32 = halves.view(np.float16).astype(np.float32)
    back = oracle.f16_to_f32(halves)
    fin = ~np.isnan(as32)
    assert np.array_equal(back[fin].view(np.uint32), as32[fin].view(np.uint32))
    # every finite half, the float just below/above it and the exact midpoints
    # between neighbouring halves, against numpy's round-to-nearest-even cast
    pos = as32[(halves < 0x7c00)]
    mids = ((pos[:-1].astype(np.float64) + pos[1:].astype(np.float64)) / 2).astype(np.float32)
    probe = np.concatenate([pos, np.nextafter(pos, np.float32(np.inf)), np.nextafter(pos, np.float32(-np.inf)),
                            mids, np.nextafter(mids, np.float32(np.inf)), np.nextafter(mids, np.float32(-np.inf))])
    probe = np.concatenate([probe, -probe, np.array([65504.0, 65519.99, 65520.0, 1e6, 1e-8, 2.0 ** -25,
                                                      np.nextafter(np.float32(2.0 ** -25), np.float32(1))],
                                                     np.float32)])
    with np.errstate(over="ignore"):
        ref = probe.astype(np.float16).view(np.uint16)
    got = oracle.f32_to_f16(probe)
    assert np.array_equal(got, ref)


# ---------------------------------------------------------------- pack
def unpack_reference(codes, gwo, perm, bits, m):
    """Independent reader of the documented layout, using Python integers."""
    n = len(bits)
    out = np.zeros((n, m), np.uint8)
    word = 0
    p = 0
    for b in (1, 2, 3, 4):
        assert gwo[b] == word
        wpr = (m * b + 31) // 32
        rows = [i for i in range(n) if bits[i] == b]
        for i in rows:
            assert perm[p] == i
            p += 1
            stream = 0
            for q in range(wpr):
                stream |= int(codes[word + q]) << (32 * q)
            for j in range(m):
                out[i, j] = (stream >> (j * b)) & ((1 << b) - 1)
            assert stream >> (m * b) == 0          # padding bits are zero
            word += wpr
    assert gwo[5] == word == len(codes)
    return out


@pytest.mark.parametrize("m", [16, 33, 100, 257])
def test_pack_round_trip_and_layout(m):
    rng = np.random.default_rng(m)
    n = 23
    bits = rng.integers(1, 5, n).astype(np.uint8)
    labels = (rng.integers(0, 16, (n, m)) % (1 << bits)[:, None]).astype(np.uint8)
    cent = rng.standard_normal((n, 16))
    W = rng.standard_normal((n, m)).astype(np.float32)
    pk = oracle.pack(W, bits, labels, cent, want_dW=True)
    assert len(pk["codes"]) == sum((m * int(b) + 31) // 32 for b in bits)
    got = unpack_reference(pk["codes"], pk["group_word_offset"], pk["row_perm"], bits, m)
    assert np.array_equal(got, labels)
    # codebooks: per row in packed order, f16(f32(centroid))
    off = 0
    for i in pk["row_perm"]:
        K = 1 << int(bits[i])
        ref = cent[i, :K].astype(np.float32).astype(np.float16).view(np.uint16)
        assert np.array_equal(pk["codebooks"][off:off + K], ref)
        # dequantised difference
        q = pk["codebooks"][off:off + K].view(np.float16).astype(np.float64)
        d = W[i].astype(np.float64) - q[labels[i]]
        assert np.array_equal(pk["dW"][i], d.astype(np.float32))   # exact difference of two floats fits fp64
        off += K
    assert off == len(pk["codebooks"])


def test_pack_known_words():
    # 3-bit row: codes 1,2,3,4,5,6,7,0,1,2,3 -> stream bits, little endian
    labels = np.array([[1, 2, 3, 4, 5, 6, 7, 0, 1, 2, 3]], np.uint8)
    bits = np.array([3], np.uint8)
    pk = oracle.pack(np.zeros((1, 11), np.float32), bits, labels, np.zeros((1, 16)))
    val = sum(int(c) << (3 * j) for j, c in enumerate(labels[0]))
    assert pk["codes"].tolist() == [val & 0xFFFFFFFF, val >> 32]
    assert pk["group_word_offset"].tolist() == [0, 0, 0, 0, 2, 2]


def test_pack_with_alpha_uses_single_rounding():
    rng = np.random.default_rng(1)
    n, m = 4, 64
    bits = np.full(n, 2, np.uint8)
    labels = rng.integers(0, 4, (n, m)).astype(np.uint8)
    cent = rng.standard_normal((n, 16)) * 0.05
    W = (rng.standard_normal((n, m)) * 0.05).astype(np.float32)
    al = skim_synth.make_alpha(0, m)
    pk = oracle.pack(W, bits, labels, cent, alpha=al, want_dW=True)
    cb = pk["codebooks"].view(np.float16).astype(np.float64).reshape(n, 4)
    # alpha (24 bits) * half (11 bits) is exact in double; the sum needs at most one
    # rounding to double which cannot straddle a float rounding boundary here except in
    # astronomically rare cases -> compare after float rounding, allow 0 mismatches
    ref = (W.astype(np.float64) - al.astype(np.float64)[None, :] * np.take_along_axis(cb, labels.astype(np.int64), 1))
    assert np.array_equal(pk["dW"], ref.astype(np.float32))


@pytest.mark.parametrize("m", [16, 33, 100, 257])
def test_unpack_and_matvec_read_back_what_pack_wrote(m):
    """The dense matrix read back from the packed model is alpha * (binary16 codebook value of the label), element
    by element (labels checked through the independent integer reader above); the product with x is the plain
    float64 matrix-vector product of that matrix."""
    rng = np.random.default_rng(100 + m)
    n = 19
    bits = rng.integers(1, 5, n).astype(np.uint8)
    labels = (rng.integers(0, 16, (n, m)) % (1 << bits)[:, None]).astype(np.uint8)
    cent = rng.standard_normal((n, 16))
    W = rng.standard_normal((n, m)).astype(np.float32)
    alpha = np.exp(rng.standard_normal(m) * 0.1).astype(np.float32)
    pk = oracle.pack(W, bits, labels, cent, alpha=alpha)
    Wq = oracle.unpack(pk["codes"], pk["group_word_offset"], pk["row_perm"], pk["codebooks"], m, alpha)
    c16 = cent.astype(np.float32).astype(np.float16).astype(np.float32)
    ref = (alpha[None, :] * np.take_along_axis(c16, labels.astype(np.int64), 1)).astype(np.float32)
    assert np.array_equal(Wq, ref)
    x = rng.standard_normal(m).astype(np.float32)
    y = oracle.dequant_matvec(pk["codes"], pk["group_word_offset"], pk["row_perm"], pk["codebooks"], m, x, alpha)
    yref = np.array([sum(float(ref[i, j]) * float(x[j]) for j in range(m)) for i in range(n)])
    np.testing.assert_allclose(y, yref, rtol=1e-12, atol=1e-12)
    # without alpha the weights are the codebook values themselves
    Wq1 = oracle.unpack(pk["codes"], pk["group_word_offset"], pk["row_perm"], pk["codebooks"], m)
    assert np.array_equal(Wq1, np.take_along_axis(c16, labels.astype(np.int64), 1))
