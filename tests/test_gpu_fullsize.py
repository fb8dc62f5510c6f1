"""GPU parity at the full sizes of the workload configs, in the launch configuration bench.py times.

Configs 1, 2 and 4: every matrix whole, every (row, bit width) entry of the error table compared with the
oracle (the oracle finishes these matrices in seconds on the machine's cores).  An entry in which the oracle met a
decision with margin < 1e-9 is excused from the exact comparison, counted against a cap measured with the
oracle on the same input, and still checked for self-consistency through the oracle's functions
(tests/parity_util.py); all other entries must match: thresholds and labels bit-exact, errors and centroids
within 1e-5 relative.  Config 3: the Hessian from all 131072 activations by the library's kernel (sampled rows
against float64), 20 iterations of the loop on a 512-row slice and one iteration on the whole layer.
"""
import numpy as np
import pytest
import torch

import oracle
import parity_util
import skim_synth

pytestmark = pytest.mark.gpu
RTOL = 1e-5
# (row, bit width) entries with a near-tie, counted by the oracle on each (config, matrix) -- 44, 191, 122, 128,
# 710, 915 -- plus a margin of about 5 %
EXCUSED_CAP = {(1, 0): 46, (2, 2): 200, (2, 0): 128, (2, 1): 135, (4, 0): 745, (4, 1): 960}


@pytest.fixture(scope="module")
def ctx(gpu_lib):
    c = gpu_lib.Context(0)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def compare_table(ctx, W, S, max_excused):
    """Whole table against the oracle, entry by entry; max_excused = the number of (row, bit width) entries in
    which the oracle meets a decision of margin < 1e-9 on this input (measured, plus a small margin)."""
    n, m = W.shape
    ref = oracle.error_table(W, S, count_near=True)
    Wd, Sd = dev(W), dev(S)
    out = ctx.error_table(Wd, Sd)
    torch.cuda.synchronize()
    E = out["E"].cpu().numpy()
    ca = out["centroids_all"].cpu().numpy()
    ua = out["upper_all"].cpu().numpy().astype(np.float64)
    st = parity_util.compare_table(W, S, None, ref, E, ca, ua)
    assert st["excused"] <= max_excused, f"{st['excused']} entries meet a near-tie, {max_excused} expected at most"
    print(f"\n[{n}x{m}] near-tie decisions init/assign = {ref['near'].tolist()}, entries excused = {st['excused']} of {E.size} "
          f"(per bit width {(~st['clean']).sum(0).tolist()}), of which {st['differ']} differ from the oracle "
          f"(largest relative gap of their errors {st['max_gap']:.2e}); max rel err E on compared entries = {st['max_rel']:.2e}")
    clean = st["clean"].all(1)
    return ref, out, clean, Wd, Sd


def check_alloc_labels_pack(ctx, gpu_lib, W, S, ref, out, clean, Wd, Sd, avg_bits, want_dW=False):
    n, m = W.shape
    E = out["E"].cpu().numpy()
    bits, spent, budget = gpu_lib.greedy_allocate(E, avg_bits)
    # the heap allocator against the linear-scan oracle on the SAME table: bit-exact
    g_same = oracle.greedy(E, avg_bits, count_near=True)
    assert np.array_equal(bits, g_same["bits"]) and spent == g_same["spent"] == budget == int(np.floor(n * avg_bits + 1e-9))
    # against the oracle's own table: differences only where excused rows changed the table
    g_ref = oracle.greedy(ref["E"], avg_bits, count_near=True)
    ndiff = int((bits != g_ref["bits"]).sum())
    assert ndiff <= 4 * int((~clean).sum()) + g_ref["near"], f"{ndiff} allocation differences"
    # the device allocator on the device table: same bits, no copy to the host
    ga = ctx.greedy_allocate_device(out["E"], avg_bits)
    torch.cuda.synchronize()
    assert np.array_equal(ga["bits"].cpu().numpy(), bits) and int(ga["info"][8]) == spent
    dbits = dev(bits)
    cr = ctx.cluster_rows(Wd, Sd, dbits)
    torch.cuda.synchronize()
    rr = oracle.cluster_rows(W, S, bits, count_near=True)
    ok = rr["near_rows"] == 0
    lab = cr["labels"].cpu().numpy()
    badl = (lab[ok] != rr["labels"][ok]).any(1)
    assert not badl.any(), f"labels differ in {int(badl.sum())} clean rows"
    assert np.all(np.abs(cr["err"].cpu().numpy()[ok] - rr["err"][ok]) <= RTOL * rr["err"][ok])
    # rows excused from the exact comparison: labels, centroids and error must still be one consistent clustering
    excused_rows = np.flatnonzero(~ok)
    parity_util.check_rows_self_consistent(W, S, None, bits, lab, cr["centroids"].cpu().numpy(),
                                           cr["upper"].cpu().numpy().astype(np.float64), cr["err"].cpu().numpy(),
                                           rows=excused_rows)
    lab_differ = int((lab[excused_rows] != rr["labels"][excused_rows]).any(1).sum())
    sel = ctx.select_allocated(dbits, out)
    pk = ctx.pack(Wd, dbits, sel["centroids"], sel["upper"], bits_host=bits, want_dW=want_dW)
    torch.cuda.synchronize()
    assert torch.equal(sel["centroids"], cr["centroids"]) and torch.equal(sel["upper"], cr["upper"])
    rp = oracle.pack(W, bits, lab, cr["centroids"].cpu().numpy(), want_dW=want_dW)
    assert np.array_equal(pk["codes"].cpu().numpy().view(np.uint32), rp["codes"])
    assert np.array_equal(pk["group_word_offset"].cpu().numpy(), rp["group_word_offset"])
    assert np.array_equal(pk["row_perm"].cpu().numpy(), rp["row_perm"])
    assert np.array_equal(pk["codebooks"].cpu().numpy().view(np.uint16), rp["codebooks"])
    if want_dW:
        assert np.array_equal(pk["dW"].cpu().numpy(), rp["dW"])
    # outputs sized for 4 bits in every row (what a caller does that never looks at the bits on the host)
    pk4 = ctx.pack(Wd, ga["bits"], sel["centroids"], sel["upper"], max_size=True)
    torch.cuda.synchronize()
    nw, ncb = len(rp["codes"]), len(rp["codebooks"])
    assert torch.equal(pk4["codes"][:nw], pk["codes"]) and torch.equal(pk4["codebooks"][:ncb], pk["codebooks"])
    assert torch.equal(pk4["group_word_offset"], pk["group_word_offset"]) and torch.equal(pk4["row_perm"], pk["row_perm"])
    print(f"[{n}x{m} @ {avg_bits}] allocation differences vs oracle table = {ndiff}, label rows excused = {int((~ok).sum())}, "
          f"of which {lab_differ} differ from the oracle")
    return bits


def test_config1_attention_projection(ctx, gpu_lib):
    W, S = skim_synth.make_ws(1)
    ref, out, clean, Wd, Sd = compare_table(ctx, W, S, max_excused=EXCUSED_CAP[(1, 0)])
    check_alloc_labels_pack(ctx, gpu_lib, W, S, ref, out, clean, Wd, Sd, 3.0)
    check_alloc_labels_pack(ctx, gpu_lib, W, S, ref, out, clean, Wd, Sd, 2.5)


def test_config2_metric_layer_down_projection(ctx, gpu_lib):
    W, S = skim_synth.make_ws(2, 2)                 # 4096 x 11008: the layer bench.py times
    ref, out, clean, Wd, Sd = compare_table(ctx, W, S, max_excused=EXCUSED_CAP[(2, 2)])
    check_alloc_labels_pack(ctx, gpu_lib, W, S, ref, out, clean, Wd, Sd, 3.2, want_dW=True)


def test_config2_metric_layer_exact_bounds(ctx, gpu_lib):
    """The two yardsticks at the size bench.py reports them: the least clustering error of every row (sampled
    rows against the oracle's O(K m^2) programme, every row against the error table it must not exceed), and the
    knapsack optimum of the allocation on the device's own table (all rows against the oracle's recurrence)."""
    W, S = skim_synth.make_ws(2, 2)
    Wd, Sd = dev(W), dev(S)
    E = ctx.error_table(Wd, Sd)["E"]
    got = ctx.kmeans_optimal(Wd, Sd)
    dp = ctx.dp_allocate(E, 3.2)
    torch.cuda.synchronize()
    E, got = E.cpu().numpy(), got.cpu().numpy()
    scale = np.sum(S.astype(np.float64) * W.astype(np.float64) ** 2, axis=1, keepdims=True)
    assert np.isfinite(got).all() and (got >= 0).all()
    assert np.all(got <= E * (1 + 1e-9) + 1e-12 * scale)
    assert np.all(np.diff(got, axis=1) <= 1e-12 * scale)
    for i in (0, 1777, 4095):
        ref = oracle.kmeans_optimal_row(W[i], S[i])
        assert np.all(np.abs(got[i] - ref) <= RTOL * ref + 1e-12 * scale[i]), (i, got[i], ref)
    ref = oracle.dp_allocate(E, 3.2)
    info = dp["info"].cpu().numpy()
    assert np.array_equal(dp["bits"].cpu().numpy(), ref["bits"])
    assert info[0] == ref["total"] and info[1] == ref["spent"] and info[2] == ref["budget"] == 13107
    g = ctx.greedy_allocate_device(dev(E), 3.2)["bits"].cpu().numpy()
    gt = E[np.arange(4096), g - 1].sum()
    assert ref["total"] <= gt
    print(f"\n[4096x11008] Lloyd / least possible error per bit width = {(E.sum(0) / got.sum(0)).round(3).tolist()}, "
          f"greedy / optimal allocation = {gt / ref['total']:.5f}")


def test_config2_joint_allocation_over_three_matrices(ctx, gpu_lib):
    """The three MLP matrices whole: both 11008 x 4096 tables entry by entry against the oracle (the 4096 x 11008
    one has its own test above and is only recomputed here), then one allocation over all 26112 rows with the
    row length as cost."""
    tables, ref_tables, costs, dirty = [], [], [], 0
    for mi in range(3):
        W, S = skim_synth.make_ws(2, mi)
        if mi < 2:
            ref, out, clean, Wd, Sd = compare_table(ctx, W, S, max_excused=EXCUSED_CAP[(2, mi)])
            ref_tables.append(ref["E"])
            dirty += int((~clean).sum())
        else:
            out = ctx.error_table(dev(W), dev(S))
            torch.cuda.synchronize()
            ref_tables.append(None)
        tables.append(out["E"].cpu().numpy())
        costs.append(np.full(W.shape[0], W.shape[1], np.int64))
        del W, S
    E = np.concatenate(tables)
    cost = np.concatenate(costs)
    bits, spent, budget = gpu_lib.greedy_allocate(E, 3.2, row_cost=cost)
    g = oracle.greedy(E, 3.2, cost=cost)
    assert np.array_equal(bits, g["bits"]) and spent == g["spent"] and budget == g["budget"]
    assert budget == int(np.floor(3.2 * cost.sum() + 1e-9)) == 432852172 and spent <= budget
    left = budget - spent
    assert all(c > left for c, b in zip(cost, bits) if b < 4)
    # per-row average (Alg. 1 as printed) on the concatenated table
    bits_u, spent_u, budget_u = gpu_lib.greedy_allocate(E, 3.2)
    assert spent_u == budget_u == int(np.floor(3.2 * len(E) + 1e-9))
    print(f"[config 2 joint] rows with an excused entry in the two tall tables: {dirty}; spent {spent} of {budget} bits")


def test_config4_tall_matrix_non_integer_budget(ctx, gpu_lib):
    W, S = skim_synth.make_ws(4, 0)                 # 22016 x 8192, whole
    ref, out, clean, Wd, Sd = compare_table(ctx, W, S, max_excused=EXCUSED_CAP[(4, 0)])
    check_alloc_labels_pack(ctx, gpu_lib, W, S, ref, out, clean, Wd, Sd, 2.25)


def test_config4_wide_matrix_rows_sorted_in_two_halves(ctx, gpu_lib):
    W, S = skim_synth.make_ws(4, 1)                 # 8192 x 22016, whole: rows longer than one LDS sort
    ref, out, clean, Wd, Sd = compare_table(ctx, W, S, max_excused=EXCUSED_CAP[(4, 1)])
    check_alloc_labels_pack(ctx, gpu_lib, W, S, ref, out, clean, Wd, Sd, 2.25)


@pytest.fixture(scope="module")
def config3_hessian(ctx):
    """H of config 3 from all 131072 synthetic activations by the library's kernel, with 64 of its rows checked
    against float64 numpy (the whole float64 product would be 2 x 10^12 operations on the host)."""
    N, m = 131072, 4096
    rows = np.random.default_rng(33).choice(m, size=64, replace=False)
    rows.sort()
    X = torch.empty((N, m), dtype=torch.bfloat16, device="cuda")
    acc = np.zeros((64, m), np.float64)
    diag = np.zeros(m, np.float64)
    done = 0
    for x in skim_synth.make_x(3, N, m, chunk=8192):
        x64 = x.astype(np.float64)
        acc += x64[:, rows].T @ x64
        diag += np.einsum("ij,ij->j", x64, x64)
        X[done:done + len(x)] = torch.from_numpy(x).cuda().to(torch.bfloat16)
        done += len(x)
    assert done == N
    H = ctx.hessian_from_activations(X)
    torch.cuda.synchronize()
    del X
    got = H[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    ref = acc / N
    d = diag / N
    scale = np.sqrt(np.outer(d[rows], d))
    worst = float((np.abs(got - ref) / scale).max())
    assert worst <= RTOL, f"H: max scaled diff {worst:.3e}"
    assert torch.equal(H, H.T.contiguous())
    print(f"\n[config 3] H from {N} activations: 64 sampled rows within {worst:.2e} of float64 (entry scale sqrt(H_jj H_ll))")
    return H


def scale_loop_iterations(ctx, W, S, Hd, H, iters, label):
    """`iters` rounds of: scale step, re-clustering at 3 bits, layer loss.  Every call is compared with the oracle
    on the GPU's own inputs (alpha, labels): labels bit-exact on rows without a near-tie and self-consistent on
    the others, loss / gradient / alpha within 1e-5."""
    n, m = W.shape
    Wd, Sd = dev(W), dev(S)
    bits = np.full(n, 3, np.uint8)
    dbits = dev(bits)
    alpha = torch.ones(m, device="cuda")
    am, av = torch.zeros(m, device="cuda"), torch.zeros(m, device="cuda")
    cr = ctx.cluster_rows(Wd, Sd, dbits, alpha=alpha)
    f32 = lambda x: float(np.float32(x))
    hp = dict(lr0=f32(0.01), beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8), decay=f32(0.5), decay_every=40)
    losses, excused = [], 0
    for it in range(1, iters + 1):
        a_in = alpha.cpu().numpy().copy()
        m_in, v_in = am.cpu().numpy().copy(), av.cpu().numpy().copy()
        lab = cr["labels"].cpu().numpy()
        o = ctx.scale_step(Wd, Sd, Hd, cr["labels"], alpha, am, av, it)
        torch.cuda.synchronize()
        ref = oracle.scale_grad(W, S, H, lab, a_in)
        assert o["loss_before"].item() == pytest.approx(ref["loss"], rel=RTOL)
        g = o["grad"].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(g - ref["grad"]) <= RTOL * np.abs(ref["grad"]) + 1e-6 * np.abs(ref["grad"]).max())
        a_ref, _, _ = oracle.adam_step(a_in, m_in, v_in, g, it, **hp)
        np.testing.assert_allclose(alpha.cpu().numpy(), a_ref, rtol=RTOL)
        a_now = alpha.cpu().numpy()
        cr = ctx.cluster_rows(Wd, Sd, dbits, alpha=alpha, out=cr)
        torch.cuda.synchronize()
        rr = oracle.cluster_rows(W, S, bits, alpha=a_now, count_near=True)
        ok = rr["near_rows"] == 0
        lab2 = cr["labels"].cpu().numpy()
        assert np.array_equal(lab2[ok], rr["labels"][ok])
        parity_util.check_rows_self_consistent(W, S, a_now, bits, lab2, cr["centroids"].cpu().numpy(),
                                               cr["upper"].cpu().numpy().astype(np.float64), cr["err"].cpu().numpy(),
                                               rows=np.flatnonzero(~ok))
        excused += int((~ok).sum())
        ll = ctx.layer_loss(Wd, Sd, Hd, cr["labels"], alpha=alpha)
        torch.cuda.synchronize()
        c2, _ = oracle.centroids_from_labels(W, S, lab2, a_now)
        rl = oracle.layer_loss(W, H, lab2, c2, a_now)
        assert ll["loss"].item() == pytest.approx(rl["loss"], rel=RTOL)
        losses.append(ll["loss"].item())
    print(f"\n[{label}] rows excused over {iters} re-clusterings: {excused}; free-running loss after each iteration: "
          + ", ".join(f"{x:.6g}" for x in losses))


def test_config3_scale_loop_20_iterations_on_a_slice(ctx, gpu_lib, config3_hessian):
    """The 20 iterations of config 3 on the first 512 rows of its layer, H from the library's kernel on all
    131072 activations."""
    W, S = skim_synth.make_ws(3, 0)
    W, S = np.ascontiguousarray(W[:512]), np.ascontiguousarray(S[:512])
    scale_loop_iterations(ctx, W, S, config3_hessian, config3_hessian.cpu().numpy(), 20, "config 3, 512 rows x 20 iterations")


def test_config3_one_iteration_on_the_whole_layer(ctx, gpu_lib, config3_hessian):
    """One iteration (step, re-clustering, loss) on all 4096 rows of the config-3 layer."""
    W, S = skim_synth.make_ws(3, 0)
    scale_loop_iterations(ctx, W, S, config3_hessian, config3_hessian.cpu().numpy(), 1, "config 3, 4096 rows x 1 iteration")


def test_config3_lfull_error_table_slice(ctx, gpu_lib, config3_hessian):
    """Layer-wise error table on a 512-row slice of the config-3 layer (H 4096 x 4096 from all 131072 synthetic
    activations): every entry of clean rows against the oracle's naive float64 dW H dW^T."""
    W, S = skim_synth.make_ws(3, 0)
    W, S = np.ascontiguousarray(W[:512]), np.ascontiguousarray(S[:512])
    n, m = W.shape
    Hd = config3_hessian
    H = Hd.cpu().numpy()
    ref = oracle.error_table_lfull(W, S, H, count_near=True)
    out = ctx.error_table_lfull(dev(W), dev(S), Hd)
    torch.cuda.synchronize()
    clean = ref["near_rows"] == 0
    assert clean.sum() >= n - 16
    got = out["E_full"].cpu().numpy()
    rel = np.abs(got[clean] - ref["E"][clean]) / ref["E"][clean]
    assert rel.max() <= RTOL, f"max rel diff {rel.max():.3e}"
    # allocation on the layer-wise table: the library's allocator and the oracle's agree on the same table
    bits, spent, budget = gpu_lib.greedy_allocate(got, 3.0)
    g = oracle.greedy(got, 3.0)
    assert np.array_equal(bits, g["bits"]) and spent == g["spent"] == budget
    print(f"\n[L-full table 512x4096] rows excused {int((~clean).sum())}, max rel err {rel.max():.2e}")


def test_joint_table_size_exact_allocation(ctx):
    """The knapsack optimum at half the rows of config 2's joint table with unit costs (13056 rows, 3.2 bits per
    row: 28723 states in 35 workgroups, 204 launches of 64 rows; the oracle's recurrence takes 12 s there and
    four times that at the full 26112) against the oracle, bit for bit; the table is synthetic (reductions of
    either sign), the clustering is not what is tested here."""
    rng = np.random.default_rng(2)
    n = 13056
    g = rng.standard_normal((n, 3)) * 0.3 + 0.5
    E = np.empty((n, 4))
    E[:, 3] = rng.random(n)
    for j in (2, 1, 0):
        E[:, j] = E[:, j + 1] + g[:, j]
    out = ctx.dp_allocate(dev(E), 3.2)
    torch.cuda.synchronize()
    ref = oracle.dp_allocate(E, 3.2)
    info = out["info"].cpu().numpy()
    assert np.array_equal(out["bits"].cpu().numpy(), ref["bits"])
    assert info[0] == ref["total"] and info[1] == ref["spent"] and info[2] == ref["budget"] == 41779
