"""Pins for the layer-loss / scale-gradient / Adam parts of the CPU oracle (no GPU)."""
import numpy as np
import pytest
import torch

import oracle
import skim_synth


def small_case(seed, n=6, m=24, K=4, with_alpha=True):
    W, S = skim_synth.make_ws_small(seed, n, m)
    S = S + np.float32(0.05)          # keep every cluster's mass away from zero
    rng = np.random.default_rng(seed)
    labels = rng.integers(0, K, (n, m)).astype(np.uint8)
    H = skim_synth.make_h_host(3, 96, m)
    al = skim_synth.make_alpha(seed, m) if with_alpha else None
    return W, S, labels, H, al


def dW_of(W, S, labels, alpha):
    c, D = oracle.centroids_from_labels(W, S, labels, alpha)
    a = np.ones(W.shape[1]) if alpha is None else alpha.astype(np.float64)
    return W.astype(np.float64) - a[None, :] * np.take_along_axis(c, labels.astype(np.int64), 1), c


def test_centroids_from_labels_are_weighted_means_in_scaled_domain():
    W, S, labels, H, al = small_case(1)
    c, D = oracle.centroids_from_labels(W, S, labels, al)
    wt = (W / al).astype(np.float64)                 # float32 ops, then widened
    st = ((S * al) * al).astype(np.float64)
    for i in range(W.shape[0]):
        for k in range(4):
            mem = labels[i] == k
            assert D[i, k] == pytest.approx(st[i, mem].sum(), rel=1e-14)
            assert c[i, k] == pytest.approx((st[i, mem] * wt[i, mem]).sum() / st[i, mem].sum(), rel=1e-13)
        assert np.all(c[i, 4:] == 0)


def test_loss_identity_hessian_is_frobenius_norm():
    W, S, labels, H, al = small_case(2)
    m = W.shape[1]
    d, c = dW_of(W, S, labels, al)
    r = oracle.layer_loss(W, np.eye(m, dtype=np.float32), labels, c, al)
    assert r["loss"] == pytest.approx((d ** 2).sum(), rel=1e-13)
    np.testing.assert_allclose(r["row_loss"], (d ** 2).sum(1), rtol=1e-13)


def test_loss_diagonal_hessian():
    W, S, labels, H, al = small_case(3)
    m = W.shape[1]
    h = np.random.default_rng(0).uniform(0.5, 2.0, m).astype(np.float32)
    d, c = dW_of(W, S, labels, al)
    r = oracle.layer_loss(W, np.diag(h), labels, c, al)
    assert r["loss"] == pytest.approx((h.astype(np.float64)[None, :] * d ** 2).sum(), rel=1e-13)


def test_loss_equals_output_error_norm():
    """tr(dW X^T X dW^T)/N = ||dW X^T||_F^2 / N (layer-wise form, Sec. 3.2 / 3.4)."""
    n, m, N = 5, 32, 64
    W, S = skim_synth.make_ws_small(4, n, m)
    labels = np.random.default_rng(4).integers(0, 8, (n, m)).astype(np.uint8)
    X = np.concatenate(list(skim_synth.make_x(3, N, m))).astype(np.float64)
    Hd = X.T @ X / N
    H = Hd.astype(np.float32)
    d, c = dW_of(W, S, labels, None)
    r = oracle.layer_loss(W, H, labels, c, None, want_P=True)
    ref = ((d @ H.astype(np.float64)) * d).sum()
    assert r["loss"] == pytest.approx(ref, rel=1e-12)
    assert r["loss"] == pytest.approx(np.linalg.norm(d @ X.T) ** 2 / N, rel=1e-6)  # H was rounded to fp32
    assert r["loss"] >= 0 and np.all(r["row_loss"] >= -1e-12)
    np.testing.assert_allclose(r["P"], d @ H.astype(np.float64), rtol=1e-12, atol=1e-15)


def test_loss_uses_H_as_written_not_transposed():
    # non-symmetric H distinguishes P = dW H from dW H^T in the returned P
    W, S, labels, H, al = small_case(5)
    m = W.shape[1]
    Hn = np.triu(np.random.default_rng(1).standard_normal((m, m))).astype(np.float32)
    d, c = dW_of(W, S, labels, al)
    r = oracle.layer_loss(W, Hn, labels, c, al, want_P=True)
    np.testing.assert_allclose(r["P"], d @ Hn.astype(np.float64), rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("seed", range(4))
def test_scale_gradient_matches_central_finite_differences(seed):
    W, S, labels, H, al = small_case(10 + seed)
    m = W.shape[1]
    g = oracle.scale_grad(W, S, H, labels, al)

    def loss_at(a64):
        # the smooth function of alpha in fp64: c = sum s a w / sum s a^2
        Wd, Sd = W.astype(np.float64), S.astype(np.float64)
        tot = 0.0
        Hd = H.astype(np.float64)
        for i in range(W.shape[0]):
            c = np.zeros(16)
            for k in range(16):
                mem = labels[i] == k
                den = (Sd[i, mem] * a64[mem] ** 2).sum()
                if den > 0:
                    c[k] = (Sd[i, mem] * a64[mem] * Wd[i, mem]).sum() / den
            d = Wd[i] - a64 * c[labels[i]]
            tot += d @ Hd @ d
        return tot

    a0 = al.astype(np.float64)
    assert g["loss"] == pytest.approx(loss_at(a0), rel=1e-12)
    fd = np.empty(m)
    for l in range(m):
        h = 1e-6
        ap, am = a0.copy(), a0.copy()
        ap[l] += h
        am[l] -= h
        fd[l] = (loss_at(ap) - loss_at(am)) / (2 * h)
    scale = np.abs(fd).max()
    np.testing.assert_allclose(g["grad"], fd, rtol=1e-6, atol=1e-7 * scale)


def test_scale_gradient_alpha_none_is_alpha_ones():
    W, S, labels, H, _ = small_case(20)
    a = oracle.scale_grad(W, S, H, labels, None)
    b = oracle.scale_grad(W, S, H, labels, np.ones(W.shape[1], np.float32))
    assert a["loss"] == b["loss"] and np.array_equal(a["grad"], b["grad"])


def test_adam_matches_torch_optimizer_with_step_decay():
    m = 50
    rng = np.random.default_rng(0)
    alpha = np.ones(m, np.float32)
    m1 = np.zeros(m, np.float32)
    m2 = np.zeros(m, np.float32)
    p = torch.nn.Parameter(torch.ones(m, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=0.01, betas=(0.9, 0.999), eps=1e-8)
    sched = torch.optim.lr_scheduler.StepLR(opt, step_size=40, gamma=0.5)
    for t in range(1, 96):
        g = rng.standard_normal(m) * (1.0 if t % 7 else 30.0)
        alpha, m1, m2 = oracle.adam_step(alpha, m1, m2, g, t)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        sched.step()
        # state is kept in float32 on the oracle side: agreement to float32 rounding
        np.testing.assert_allclose(alpha, p.detach().numpy(), rtol=3e-6)
    assert sched.get_last_lr()[0] == pytest.approx(0.0025)


def test_adam_first_step_moves_by_lr_against_gradient_sign():
    g = np.array([3.0, -0.02, 1e-3, -7.0])
    a, m1, m2 = oracle.adam_step(np.ones(4, np.float32), np.zeros(4, np.float32), np.zeros(4, np.float32), g, 1)
    np.testing.assert_allclose(a, 1.0 - 0.01 * np.sign(g), rtol=1e-5)
    np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-6)
    np.testing.assert_allclose(m2, 0.001 * g * g, rtol=1e-6)


def test_lfull_error_table_reduces_to_sdiag_when_hessian_is_diagonal():
    """Sec. 3.4: with H = diag(h) the layer-wise error of channel i is sum_j h_j dW_ij^2; if every
    channel's sensitivity row equals h this is the S-diag objective the K-means minimises, so the two
    tables coincide (a dropped row, a transposed H or labels of the wrong bit width would break it)."""
    n, m = 12, 96
    W, _ = skim_synth.make_ws_small(11, n, m)
    rng = np.random.default_rng(5)
    h = (rng.standard_normal(m) ** 2 + 0.01).astype(np.float32)
    S = np.tile(h, (n, 1))
    full = oracle.error_table_lfull(W, S, np.diag(h).astype(np.float32))
    sdiag = oracle.error_table(W, S)
    np.testing.assert_allclose(full["E"], sdiag["E"], rtol=1e-12)


def test_lfull_error_table_by_definition_on_a_tiny_case():
    """Brute force: E[i][b] = sum_jl dW_ij H_jl dW_il with dW from the labels and centroids of the b-bit clustering."""
    n, m = 5, 32
    W, S = skim_synth.make_ws_small(12, n, m)
    H = skim_synth.make_h_host(3, 64, m).astype(np.float64)
    al = skim_synth.make_alpha(4, m)
    full = oracle.error_table_lfull(W, S, H.astype(np.float32), alpha=al)
    for b in (1, 2, 3, 4):
        cr = oracle.cluster_rows(W, S, np.full(n, b, np.uint8), alpha=al)
        d = W.astype(np.float64) - al.astype(np.float64)[None, :] * np.take_along_axis(cr["centroids"], cr["labels"].astype(np.int64), 1)
        ref = np.einsum("ij,jl,il->i", d, H.astype(np.float32).astype(np.float64), d)
        np.testing.assert_allclose(full["E"][:, b - 1], ref, rtol=1e-12)


def test_train_scale_decreases_the_layer_loss_and_returns_consistent_pieces():
    """Alg. 2 as a whole on a tiny layer: the loss trace is the loss at each alpha visited (checked against
    layer_loss directly), Adam with these step sizes lowers it, and the returned centroids are the weighted
    means of the returned labels at the returned alpha."""
    n, m = 8, 48
    W, S = skim_synth.make_ws_small(31, n, m)
    S = S + np.float32(0.05)
    H = skim_synth.make_h_host(3, 192, m)
    bits = np.full(n, 2, np.uint8)
    r = oracle.train_scale(W, S, H, bits, np.ones(m, np.float32), steps=25)
    assert len(r["loss_trace"]) == 26
    assert r["loss_trace"][-1] < r["loss_trace"][0]
    c, _ = oracle.centroids_from_labels(W, S, r["labels"], r["alpha"])
    np.testing.assert_array_equal(c, r["centroids"])
    assert r["loss_trace"][-1] == pytest.approx(oracle.layer_loss(W, H, r["labels"], c, r["alpha"])["loss"], rel=1e-13)
    # first entry: loss of the plain clustering at alpha = 1
    cr = oracle.cluster_rows(W, S, bits)
    c0, _ = oracle.centroids_from_labels(W, S, cr["labels"], None)
    assert r["loss_trace"][0] == pytest.approx(oracle.layer_loss(W, H, cr["labels"], c0, None)["loss"], rel=1e-13)
    # step numbering: two rounds of 10 steps from t0 = 1 equal the manual composition
    r2 = oracle.train_scale(W, S, H, bits, np.ones(m, np.float32), steps=3, outer=2)
    assert len(r2["loss_trace"]) == 7


def test_hessian_from_activations_by_definition():
    """H_jl = (1/N) sum_k x_kj x_kl, checked entry by entry with Python floats; symmetric, and the layer loss
    written with H equals the mean squared output error ||X dW^T||^2 / N (Sec. 3.4)."""
    N, m = 40, 12
    X = np.concatenate(list(skim_synth.make_x(3, N, m)))
    H = oracle.hessian_from_activations(X)
    for j in range(m):
        for l in range(m):
            ref = sum(float(X[k, j]) * float(X[k, l]) for k in range(N)) / N
            assert H[j, l] == np.float32(ref)
    assert np.array_equal(H, H.T)
    rng = np.random.default_rng(1)
    d = rng.standard_normal((3, m))
    out_err = ((X.astype(np.float64) @ d.T) ** 2).sum(0) / N
    np.testing.assert_allclose(np.einsum("ij,jl,il->i", d, H.astype(np.float64), d), out_err, rtol=1e-6)
