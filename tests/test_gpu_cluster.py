"""GPU parity: clustering, error table, allocation and packing against the CPU oracle.

Bar: labels, thresholds, allocations, packed codes and codebooks bit-exact;
centroids and errors within 1e-5 relative (the benchmark spec).  A decision whose oracle
margin is below 1e-9 may legitimately fall the other way (the two sides sum in
different orders); the oracle counts such decisions per (row, bit width), only
those entries are excused from the exact comparison, and they are still checked
for self-consistency through the oracle's functions (tests/parity_util.py).
On config 0 the count must be zero.
"""
import numpy as np
import pytest
import torch

import oracle
import parity_util
import skim_synth

pytestmark = pytest.mark.gpu

RTOL = 1e-5


@pytest.fixture(scope="module")
def ctx(gpu_lib):
    c = gpu_lib.Context(0)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_close(got, ref, rtol=RTOL):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    scale = np.maximum(np.abs(ref), 1e-300)
    return np.abs(got - ref) <= rtol * scale + 0.0


def check_table(ctx, W, S, alpha=None, iters=30, bmin=1, bmax=4, require_no_near=False):
    """Error table against the oracle, entry by entry (parity_util.compare_table).  Returns the oracle's result,
    the GPU's, and the number of (row, bit width) entries excused from the exact comparison."""
    ref = oracle.error_table(W, S, alpha, bmin=bmin, bmax=bmax, T=iters, count_near=True)
    out = ctx.error_table(dev(W), dev(S), None if alpha is None else dev(alpha), bmin=bmin, bmax=bmax, iters=iters)
    torch.cuda.synchronize()
    E = out["E"].cpu().numpy()
    ca = out["centroids_all"].cpu().numpy()
    ua = out["upper_all"].cpu().numpy()
    if require_no_near:
        assert ref["near"].tolist() == [0, 0]
    st = parity_util.compare_table(W, S, alpha, ref, E, ca, ua, bmin=bmin, bmax=bmax)
    return ref, out, st["excused"]


def check_rows(ctx, W, S, bits, alpha=None, iters=30):
    """cluster_rows against the oracle: rows without a near-tie bit-exact (labels, thresholds), the others a
    consistent clustering of their own (labels follow from the thresholds, centroids and error from the labels)."""
    cr = ctx.cluster_rows(dev(W), dev(S), dev(bits), alpha=None if alpha is None else dev(alpha), iters=iters)
    torch.cuda.synchronize()
    rr = oracle.cluster_rows(W, S, bits, alpha=alpha, T=iters, count_near=True)
    clean = rr["near_rows"] == 0
    lab = cr["labels"].cpu().numpy()
    up = cr["upper"].cpu().numpy().astype(np.float64)
    assert np.array_equal(lab[clean], rr["labels"][clean])
    assert np.array_equal(up[clean], rr["upper"][clean])
    parity_util.check_rows_self_consistent(W, S, alpha, bits, lab, cr["centroids"].cpu().numpy(), up,
                                           cr["err"].cpu().numpy(), rows=np.flatnonzero(~clean))
    return cr, rr, clean


def test_config0_error_table_allocation_labels_and_pack(ctx, gpu_lib):
    W, S = skim_synth.make_ws(0)
    ref, out, excused = check_table(ctx, W, S, require_no_near=True)
    assert excused == 0
    E = out["E"].cpu().numpy()
    # allocation to 3.0 bits through the library's allocator on the GPU's table
    bits, spent, budget = gpu_lib.greedy_allocate(E, 3.0)
    g = oracle.greedy(ref["E"], 3.0, count_near=True)
    assert g["near"] == 0
    assert np.array_equal(bits, g["bits"]) and spent == g["spent"] == 1536 and budget == 1536
    # K-means at the allocated widths: labels bit-exact
    dbits = dev(bits)
    cr = ctx.cluster_rows(dev(W), dev(S), dbits)
    torch.cuda.synchronize()
    rr = oracle.cluster_rows(W, S, bits, count_near=True)
    assert int(rr["near_rows"].sum()) == 0
    assert np.array_equal(cr["labels"].cpu().numpy(), rr["labels"])
    assert np.array_equal(cr["upper"].cpu().numpy().astype(np.float64), rr["upper"])
    assert rel_close(cr["err"].cpu().numpy(), rr["err"]).all()
    np.testing.assert_allclose(cr["centroids"].cpu().numpy(), rr["centroids"], rtol=RTOL, atol=1e-14)
    # the per-bit blocks of the table hold the same clustering (no second K-means needed)
    sel = ctx.select_allocated(dbits, out)
    torch.cuda.synchronize()
    assert torch.equal(sel["centroids"], cr["centroids"]) and torch.equal(sel["upper"], cr["upper"])
    assert torch.equal(sel["err"], cr["err"])
    # pack from thresholds
    pk = ctx.pack(dev(W), dbits, sel["centroids"], sel["upper"], want_dW=True, bits_host=bits)
    torch.cuda.synchronize()
    rp = oracle.pack(W, bits, rr["labels"], rr["centroids"], want_dW=True)
    assert np.array_equal(pk["codes"].cpu().numpy().view(np.uint32), rp["codes"])
    assert np.array_equal(pk["group_word_offset"].cpu().numpy(), rp["group_word_offset"])
    assert np.array_equal(pk["row_perm"].cpu().numpy(), rp["row_perm"])
    assert np.array_equal(pk["codebooks"].cpu().numpy().view(np.uint16), rp["codebooks"])
    assert np.array_equal(pk["dW"].cpu().numpy(), rp["dW"])


@pytest.mark.parametrize("m", [16, 17, 33, 100, 255, 256, 257, 1000, 2049, 4095, 4097])
def test_ragged_row_lengths(ctx, m):
    W, S = skim_synth.make_ws_small(m, 24, m)
    ref, out, excused = check_table(ctx, W, S)
    assert excused <= 1


@pytest.mark.parametrize("m", [16385, 16400, 20000, 32768])
def test_rows_longer_than_one_lds_sort(ctx, m):
    W, S = skim_synth.make_ws_small(m, 6, m, dup_frac=0.05)
    S[2] = 0.0                      # no sensitivity mass: unit weights on the merged path too
    W[3, : m // 2] = np.sort(W[3, : m // 2])        # first half entirely below / interleaved with the second
    ref, out, excused = check_table(ctx, W, S)
    assert excused <= 6          # entries, as counted by the oracle on these inputs (2, 3, 6, 4)
    bits = np.array([1, 2, 3, 4, 3, 2], np.uint8)
    check_rows(ctx, W, S, bits)


def test_duplicates_zero_sensitivities_and_dead_rows(ctx):
    W, S = skim_synth.make_ws_small(7, 64, 300, dup_frac=0.3, zero_s_frac=0.4)
    S[3] = 0.0                      # a row without any sensitivity mass -> unit weights
    W[5] = np.float32(0.25)         # a constant row: every cluster but the first is empty
    W[6, :150] = np.float32(-1.0)   # two distinct values only
    W[6, 150:] = np.float32(2.0)
    W[7] = np.round(W[7] * 200) / 200   # few distinct values, many exact ties in the sort
    W[8, ::2] = 0.0
    W[8, 1::4] = -0.0               # both zeros are one value
    ref, out, excused = check_table(ctx, W, S)
    assert excused <= 4          # rows of few distinct values put elements exactly between two centroids
    bits = (np.arange(64) % 4 + 1).astype(np.uint8)
    check_rows(ctx, W, S, bits)


def test_heavy_element_rows_exercise_rank_repair(ctx):
    W, S = skim_synth.make_ws_small(9, 32, 500)
    S[np.arange(32), np.arange(32) * 13 % 500] = 1e9     # one element carries nearly all mass
    S[4, -1] = 1e12
    S[5, np.argmax(W[5])] = 1e12                          # the largest element: ranks are pushed down
    S[6, np.argmin(W[6])] = 1e12
    ref, out, excused = check_table(ctx, W, S)
    assert excused <= 1


@pytest.mark.parametrize("iters", [1, 2, 7])
def test_iteration_counts(ctx, iters):
    W, S = skim_synth.make_ws_small(40 + iters, 40, 777)
    check_table(ctx, W, S, iters=iters)


def test_bit_range_subset(ctx):
    W, S = skim_synth.make_ws_small(50, 16, 400)
    check_table(ctx, W, S, bmin=2, bmax=3)
    check_table(ctx, W, S, bmin=4, bmax=4)
    check_table(ctx, W, S, bmin=1, bmax=1)


def test_scaled_clustering(ctx):
    W, S = skim_synth.make_ws_small(60, 48, 640)
    al = skim_synth.make_alpha(3, 640, spread=0.2)
    ref, out, excused = check_table(ctx, W, S, alpha=al)
    assert excused <= 1
    bits = np.full(48, 3, np.uint8)
    cr, rr, clean = check_rows(ctx, W, S, bits, alpha=al)
    # pack with alpha: thresholds live in the scaled domain
    pk = ctx.pack(dev(W), dev(bits), cr["centroids"], cr["upper"], alpha=dev(al), want_dW=True, bits_host=bits)
    torch.cuda.synchronize()
    if clean.all():
        rp = oracle.pack(W, bits, rr["labels"], rr["centroids"], alpha=al, want_dW=True)
        assert np.array_equal(pk["codes"].cpu().numpy().view(np.uint32), rp["codes"])
        assert np.array_equal(pk["codebooks"].cpu().numpy().view(np.uint16), rp["codebooks"])
        assert np.array_equal(pk["dW"].cpu().numpy(), rp["dW"])


def test_row_stride(ctx):
    W, S = skim_synth.make_ws_small(70, 20, 512)
    Wd, Sd = dev(W), dev(S)
    out = ctx.error_table(Wd[:, :300], Sd[:, :300])       # ld = 512, m = 300
    torch.cuda.synchronize()
    ref = oracle.error_table(W[:, :300], S[:, :300], count_near=True)
    clean = ref["near_rows"] == 0
    assert rel_close(out["E"].cpu().numpy()[clean], ref["E"][clean]).all()


def test_many_rows_of_repeated_values_take_the_network_row_after_row(ctx):
    """Every row holds 24 distinct weights, each about ten times over (4 to 20 times): the value bins of the sort
    overflow in every row, so every row of a workgroup is attempted by the bucket path and then either finished by
    its third pass or dropped and sorted by the network (there are many more rows than resident workgroups).
    Results must not depend on which path sorted a row or on what the row before it left behind."""
    n, m = 30000, 256
    rng = np.random.default_rng(77)
    vals = (rng.standard_normal((n, 24)) * 0.02).astype(np.float32)
    pick = rng.integers(0, 24, (n, m))
    W = np.take_along_axis(vals, pick, axis=1)
    S = (rng.standard_normal((n, m)) ** 2).astype(np.float32)
    rows = np.r_[0:64, 14000:14064, n - 64:n]      # the oracle's comparison on a sample of rows, the GPU on all
    out = ctx.error_table(dev(W), dev(S))
    torch.cuda.synchronize()
    ref = oracle.error_table(W[rows], S[rows], count_near=True)
    E = out["E"].cpu().numpy()[rows]
    ca = out["centroids_all"].cpu().numpy()[rows]
    ua = out["upper_all"].cpu().numpy()[rows]
    st = parity_util.compare_table(W[rows], S[rows], None, ref, E, ca, ua)
    assert st["clean"].mean() > 0.5, "too few entries compared exactly"
    # the same rows on their own (one row per workgroup: the first attempt of the bucket path, then the network)
    alone = ctx.error_table(dev(W[rows]), dev(S[rows]))
    torch.cuda.synchronize()
    assert np.array_equal(alone["E"].cpu().numpy(), E)
    assert np.array_equal(alone["upper_all"].cpu().numpy(), ua)
    assert np.array_equal(alone["centroids_all"].cpu().numpy(), ca)


@pytest.mark.parametrize("where", ["start", "middle", "end"])
@pytest.mark.parametrize("m", [1000, 4096, 11008])
def test_rows_with_one_value_9_to_20_times_over(ctx, m, where):
    """Smooth rows in which one value occurs k times, k = 9 .. 20, starting at every alignment to the sort's
    16-slot windows (the rank of the repeated value moves from row to row; at either end of the row or in the
    middle): the value's bin holds k keys, more than
    the two register passes of the bucket path put in order (9 they still do).  Up to 17 the third pass finishes the row, beyond
    that the network does; either way the table must be the oracle's."""
    rng = np.random.default_rng(4100 + m + len(where))
    ks = list(range(9, 21))
    n = len(ks) * 16
    W = (rng.standard_normal((n, m)) * 0.02).astype(np.float32)
    S = (rng.standard_normal((n, m)) ** 2).astype(np.float32)
    for i in range(n):
        k = ks[i // 16]
        order = np.argsort(W[i], kind="stable")
        # rank at which the run of equal values starts: at the least weights of the row, in the middle, or so that
        # the run ends within the last 16 ranks (the last, possibly part-filled, window of the sort)
        r = {"start": i % 16, "middle": (m // 3) + (i % 16), "end": m - k - (i % 16)}[where]
        cols = order[r:r + k]
        W[i, cols] = W[i, order[r]]
    ref, out, excused = check_table(ctx, W, S)
    assert excused <= n // 8


@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
def test_weights_converted_from_a_16_bit_format(ctx, fmt):
    """Weights that were rounded to bfloat16 / float16 and widened again: every row holds each value many times
    over, and the sort spreads equal weights over its value bins by their sensitivity.  Rows long enough to fill
    the bins, more rows than workgroups (so that the carried bin map is exercised), oracle on a sample of rows."""
    n, m = 600, 11008
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((n, m)) * 0.02).astype(np.float32)
    mask = rng.random((n, m)) < 0.005
    W = np.where(mask, (rng.standard_normal((n, m)) * 0.2).astype(np.float32), W)
    if fmt == "bf16":
        W = torch.from_numpy(W).bfloat16().float().numpy()
    else:
        W = W.astype(np.float16).astype(np.float32)
    S = (rng.standard_normal((n, m)) ** 2).astype(np.float32)
    S[5, ::3] = 0.0                                   # sensitivities with exact zeros in one row
    W[7] = -np.abs(W[7])                              # a row of negative weights only
    out = ctx.error_table(dev(W), dev(S))
    torch.cuda.synchronize()
    rows = np.r_[0:24, 300:316, n - 8:n]
    ref = oracle.error_table(W[rows], S[rows], count_near=True)
    st = parity_util.compare_table(W[rows], S[rows], None, ref, out["E"].cpu().numpy()[rows],
                                   out["centroids_all"].cpu().numpy()[rows], out["upper_all"].cpu().numpy()[rows])
    # (repeated values make exact ties common: the oracle excuses most entries above one bit, and those are held
    # to the self-consistency checks; the one-bit entries and the rest are compared exactly)
    assert st["clean"].mean() > 0.1, "too few entries compared exactly"
    bits = rng.integers(1, 5, len(rows)).astype(np.uint8)
    check_rows(ctx, W[rows], S[rows], bits)


def test_pack_mixed_bits_matches_oracle_layout(ctx):
    n, m = 97, 1111
    W, S = skim_synth.make_ws_small(80, n, m)
    bits = np.random.default_rng(0).integers(1, 5, n).astype(np.uint8)
    cr = ctx.cluster_rows(dev(W), dev(S), dev(bits))
    torch.cuda.synchronize()
    rr = oracle.cluster_rows(W, S, bits, count_near=True)
    pk = ctx.pack(dev(W), dev(bits), cr["centroids"], cr["upper"], bits_host=bits)
    torch.cuda.synchronize()
    # pack is compared on the GPU's own labels (isolates the packer from clustering near-ties)
    rp = oracle.pack(W, bits, cr["labels"].cpu().numpy(), cr["centroids"].cpu().numpy())
    assert np.array_equal(pk["codes"].cpu().numpy().view(np.uint32), rp["codes"])
    assert np.array_equal(pk["group_word_offset"].cpu().numpy(), rp["group_word_offset"])
    assert np.array_equal(pk["row_perm"].cpu().numpy(), rp["row_perm"])
    assert np.array_equal(pk["codebooks"].cpu().numpy().view(np.uint16), rp["codebooks"])
    clean = rr["near_rows"] == 0
    assert np.array_equal(cr["labels"].cpu().numpy()[clean], rr["labels"][clean])


def test_validation_mode_reports_values_the_method_is_undefined_on(gpu_lib):
    W, S = skim_synth.make_ws_small(91, 6, 200)
    al = skim_synth.make_alpha(2, 200)
    c = gpu_lib.Context(0)
    try:
        c.validate_enable(True)
        c.error_table(dev(W), dev(S), dev(al))                      # clean inputs pass
        for arr, name, val in [("W", "W", np.nan), ("W", "W", np.inf), ("S", "S", -1.0), ("S", "S", np.nan),
                               ("alpha", "alpha", 0.0), ("alpha", "alpha", -np.inf)]:
            Wb, Sb, ab = W.copy(), S.copy(), al.copy()
            {"W": Wb, "S": Sb, "alpha": ab}[arr].flat[137] = val
            with pytest.raises(gpu_lib.SkimError, match=name) as ei:
                c.error_table(dev(Wb), dev(Sb), dev(ab))
            assert ei.value.status == -6
        with pytest.raises(gpu_lib.SkimError):
            Sb = S.copy()
            Sb[5, 199] = -0.5                                       # the last element of the last row
            c.cluster_rows(dev(W), dev(Sb), dev(np.full(6, 2, np.uint8)))
        c.validate_enable(False)
        Sb = S.copy()
        Sb[0, 0] = -1.0
        c.error_table(dev(W), dev(Sb))                              # off (the default): not looked for, no error
        torch.cuda.synchronize()
    finally:
        c.close()


def test_argument_errors(ctx, gpu_lib):
    W, S = skim_synth.make_ws_small(90, 4, 64)
    with pytest.raises(gpu_lib.SkimError):
        ctx.error_table(dev(W)[:, :8], dev(S)[:, :8])              # m < 2^bmax
    with pytest.raises(gpu_lib.SkimError):
        ctx.error_table(dev(W), dev(S), bmin=0)
    with pytest.raises(gpu_lib.SkimError):
        ctx.error_table(dev(W), dev(S), iters=0)
    big = torch.zeros((1, gpu_lib.MAX_M + 1), dtype=torch.float32, device="cuda")
    with pytest.raises(gpu_lib.SkimError):
        ctx.error_table(big, big)
    with pytest.raises(gpu_lib.SkimError):
        gpu_lib.greedy_allocate(np.zeros((4, 4)), 5.0)


@pytest.mark.parametrize("n,m,with_alpha", [(37, 100, False), (64, 257, True), (130, 1500, True), (16, 11008, False),
                                            (3, 16, True), (9, 4096, True)])
def test_unpack_and_dequant_matvec_match_oracle(ctx, gpu_lib, n, m, with_alpha):
    """The packed model read back on the GPU: dense weights bit-exact, matrix-vector product (float64
    accumulation, different summation order) to 1e-12 of the sum of magnitudes."""
    W, S = skim_synth.make_ws_small(77, n, m)
    al = skim_synth.make_alpha(5, m) if with_alpha else None
    rng = np.random.default_rng(n * 1000 + m)
    bits = rng.integers(1, 5, n).astype(np.uint8)
    Wd, Sd, bd = dev(W), dev(S), dev(bits)
    ald = None if al is None else dev(al)
    cr = ctx.cluster_rows(Wd, Sd, bd, alpha=ald)
    pk = ctx.pack(Wd, bd, cr["centroids"], cr["upper"], alpha=ald, bits_host=bits)
    x = rng.standard_normal(m).astype(np.float32)
    Wq = ctx.unpack(pk, m, alpha=ald)
    y = ctx.dequant_matvec(pk, m, dev(x), alpha=ald)
    torch.cuda.synchronize()
    args = (pk["codes"].cpu().numpy().view(np.uint32), pk["group_word_offset"].cpu().numpy(),
            pk["row_perm"].cpu().numpy(), pk["codebooks"].cpu().numpy().view(np.uint16), m)
    ref = oracle.unpack(*args, alpha=al)
    assert np.array_equal(Wq.cpu().numpy(), ref)
    yref = oracle.dequant_matvec(*args, x, alpha=al)
    scale = np.abs(ref.astype(np.float64)) @ np.abs(x.astype(np.float64))
    assert np.all(np.abs(y.cpu().numpy() - yref) <= 1e-12 * scale)
    # the float32 reader: same product, float32 fused multiply-adds in its own order
    yf = ctx.dequant_matvec_f32(pk, m, dev(x), alpha=ald)
    torch.cuda.synchronize()
    assert np.all(np.abs(yf.cpu().numpy().astype(np.float64) - yref) <= 1e-5 * scale)
    # x at an address that is no multiple of 16: the kernel with 4-byte loads
    xo = torch.zeros(m + 1, dtype=torch.float32, device="cuda")
    xo[1:] = dev(x)
    y2 = ctx.dequant_matvec(pk, m, xo[1:], alpha=ald)
    yf2 = ctx.dequant_matvec_f32(pk, m, xo[1:], alpha=ald)
    torch.cuda.synchronize()
    assert np.all(np.abs(y2.cpu().numpy() - yref) <= 1e-12 * scale)
    assert np.all(np.abs(yf2.cpu().numpy().astype(np.float64) - yref) <= 1e-5 * scale)


def _tables(rng, n, kind):
    if kind == "smooth":
        g = np.sort(rng.random((n, 3)), axis=1)[:, ::-1] * rng.random((n, 1))
    elif kind == "ties":
        g = rng.integers(0, 4, (n, 3)).astype(np.float64)          # many equal reductions, some zero
    elif kind == "nonmonotone":
        g = rng.standard_normal((n, 3))                            # reductions of any sign and order
    else:
        g = np.zeros((n, 3))
    E = np.empty((n, 4))
    E[:, 3] = rng.random(n)
    for j in (2, 1, 0):
        E[:, j] = E[:, j + 1] + g[:, j]
    return E


@pytest.mark.parametrize("kind", ["smooth", "ties", "nonmonotone", "flat"])
@pytest.mark.parametrize("n,avg", [(1, 2.0), (7, 1.0), (7, 4.0), (100, 2.5), (1000, 3.2), (4096, 3.2), (22016, 2.25)])
def test_device_greedy_equals_host_and_oracle(ctx, gpu_lib, kind, n, avg):
    """Alg. 1 on the device: same bits as the host function and as the oracle's linear-scan loop on the same
    table, including tables full of ties, reductions of either sign, and the two ends of the budget."""
    rng = np.random.default_rng(n * 7 + len(kind))
    E = _tables(rng, n, kind)
    out = ctx.greedy_allocate_device(dev(E), avg)
    torch.cuda.synchronize()
    bits_h, spent, budget = gpu_lib.greedy_allocate(E, avg)
    got = out["bits"].cpu().numpy()
    info = out["info"].cpu().numpy()
    assert np.array_equal(got, bits_h)
    assert info[8] == spent == budget == info[9]
    assert np.array_equal(info[:8], np.bincount(bits_h, minlength=8))
    if n <= 4096:
        assert np.array_equal(got, oracle.greedy(E, avg)["bits"])


@pytest.mark.parametrize("kind", ["smooth", "ties", "nonmonotone", "flat"])
@pytest.mark.parametrize("n,avg,bmin,bmax", [(1, 2.0, 1, 4), (7, 1.0, 1, 4), (7, 4.0, 1, 4), (100, 2.5, 1, 4),
                                             (129, 3.2, 1, 4), (1000, 3.2, 1, 4), (4096, 3.2, 1, 4),
                                             (3000, 3.999, 1, 4), (5000, 3.4, 3, 4), (300, 2.5, 2, 3)])
def test_dp_allocation_equals_oracle(ctx, kind, n, avg, bmin, bmax):
    """The exact allocation: same bits, same total, same spent bits as the oracle's recurrence (same order of
    additions and the same tie rules, so nothing is left to rounding).  The sizes put the states in one
    workgroup (n <= 2600 at three extra bits) and in several, and the rows in one launch and in many."""
    rng = np.random.default_rng(n * 11 + len(kind))
    E = np.ascontiguousarray(_tables(rng, n, kind)[:, bmin - 1:bmax])
    out = ctx.dp_allocate(dev(E), avg, bmin=bmin, bmax=bmax)
    torch.cuda.synchronize()
    ref = oracle.dp_allocate(E, avg, bmin=bmin, bmax=bmax)
    info = out["info"].cpu().numpy()
    assert np.array_equal(out["bits"].cpu().numpy(), ref["bits"])
    assert info[0] == ref["total"] and info[1] == ref["spent"] and info[2] == ref["budget"]
    if kind in ("smooth",):
        # reductions that shrink with the bits: Alg. 1 reaches the same optimum
        g = ctx.greedy_allocate_device(dev(E), avg, bmin=bmin, bmax=bmax)
        gb = g["bits"].cpu().numpy()
        tot = E[np.arange(n), gb - bmin].sum()
        assert tot == pytest.approx(ref["total"], rel=1e-12)


def test_dp_allocation_rejects_bad_arguments(ctx):
    E = dev(np.zeros((10, 4)))
    with pytest.raises(Exception):
        ctx.dp_allocate(E, 0.5)
    with pytest.raises(Exception):
        ctx.dp_allocate(E, 4.5)
    assert ctx.lib.skim_dp_allocate_scratch_bytes(10, 1, 6, 2.0) == 0      # more than three bits apart
    out = ctx.dp_allocate(E, 2.0)
    torch.cuda.synchronize()
    assert np.all(out["bits"].cpu().numpy() == 1) and out["info"][0].item() == 0.0   # nothing to gain: no bit spent


def _optimal_close(got, ref, W, S, alpha=None):
    """An entry is a difference of float64 prefix sums of s w^2: absolute error of a few ulps of the row's whole
    second moment, on top of the relative tolerance of the other floating-point outputs."""
    scale = np.empty(W.shape[0])
    for i in range(W.shape[0]):
        w, s = (W[i], S[i]) if alpha is None else oracle.scale_row(W[i], S[i], alpha)
        s = s.astype(np.float64) if np.any(s > 0) else np.ones(len(s))
        scale[i] = np.sum(s * w.astype(np.float64) ** 2)
    return np.abs(got - ref) <= RTOL * np.abs(ref) + 1e-12 * scale[:, None], scale[:, None]


@pytest.mark.parametrize("n,m,dup,zs", [(24, 16, 0.0, 0.0), (24, 100, 0.2, 0.3), (20, 257, 0.0, 0.0), (12, 1000, 0.05, 0.1),
                                        (6, 2049, 0.0, 0.0)])
def test_optimal_clustering_error_matches_oracle(ctx, n, m, dup, zs):
    """The exact floor of the clustering error against the oracle's O(K m^2) programme (the GPU fills each layer
    by halving with the monotone-cut bounds): same values, and never above what the Lloyd iterations reach."""
    W, S = skim_synth.make_ws_small(m + n, n, m, dup_frac=dup, zero_s_frac=zs)
    S[1] = 0.0                                   # no mass: unit weights
    W[2] = np.float32(0.5)                       # one value: nothing to lose
    W[3] = np.round(W[3] * 50) / 50              # few distinct values
    got = ctx.kmeans_optimal(dev(W), dev(S))
    table = ctx.error_table(dev(W), dev(S))["E"]
    torch.cuda.synchronize()
    got, table = got.cpu().numpy(), table.cpu().numpy()
    ref = oracle.kmeans_optimal_table(W, S)
    close, scale = _optimal_close(got, ref, W, S)
    assert np.all(close)
    assert np.all(got[2] <= 1e-12 * scale[2]) and np.all(np.diff(got, axis=1) <= 1e-12 * scale)
    assert np.all(got <= table * (1 + 1e-9) + 1e-12 * scale)


def test_optimal_clustering_error_scaled_inputs_and_bit_subset(ctx):
    W, S = skim_synth.make_ws_small(77, 16, 300)
    rng = np.random.default_rng(5)
    alpha = rng.uniform(0.5, 2.0, 300).astype(np.float32)
    got = ctx.kmeans_optimal(dev(W), dev(S), alpha=dev(alpha), bmin=2, bmax=3)
    torch.cuda.synchronize()
    ref = oracle.kmeans_optimal_table(W, S, alpha=alpha, bmin=2, bmax=3)
    assert got.shape == (16, 2) and np.all(_optimal_close(got.cpu().numpy(), ref, W, S, alpha)[0])


@pytest.mark.parametrize("m,bmax", [(14000, 1), (16400, 2)])
def test_optimal_clustering_error_long_rows(ctx, m, bmax):
    """Rows too long for the cuts to sit in LDS (they move to the caller's scratch), and rows sorted in two halves."""
    W, S = skim_synth.make_ws_small(m, 2, m, dup_frac=0.02)
    got = ctx.kmeans_optimal(dev(W), dev(S), bmin=1, bmax=bmax)
    torch.cuda.synchronize()
    ref = oracle.kmeans_optimal_table(W, S, bmin=1, bmax=bmax)
    close, _ = _optimal_close(got.cpu().numpy(), ref, W, S)
    assert np.all(close)


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_and_flavours(ctx, seed):
    """Seeded sweep over combinations the targeted tests cover one at a time: row count (odd and even: two rows
    share a wavefront), ragged length, duplicated values, zero sensitivities, heavy elements, column scaling,
    iteration count and bit range."""
    rng = np.random.default_rng(9000 + seed)
    n = int(rng.integers(1, 48))
    m = int(rng.choice([16, 31, 64, 100, 333, 1024, 1500, 3001, 5000]))
    W, S = skim_synth.make_ws_small(500 + seed, n, m, dup_frac=float(rng.choice([0.0, 0.1, 0.5])),
                                    zero_s_frac=float(rng.choice([0.0, 0.2, 0.9])))
    if seed % 3 == 0:
        S[np.arange(n), rng.integers(0, m, n)] = 1e8                 # one element carries the mass
    if seed % 4 == 1:
        S[rng.integers(0, n)] = 0.0                                  # a row without mass
    alpha = rng.uniform(0.5, 2.0, m).astype(np.float32) if seed % 2 else None
    bmin = int(rng.integers(1, 4))
    bmax = int(rng.integers(bmin, 5))
    iters = int(rng.choice([1, 3, 30]))
    ref, out, excused = check_table(ctx, W, S, alpha=alpha, iters=iters, bmin=bmin, bmax=bmax)
    assert excused <= 2
    bits = rng.integers(1, 5, n).astype(np.uint8)
    check_rows(ctx, W, S, bits, alpha=alpha, iters=iters)
