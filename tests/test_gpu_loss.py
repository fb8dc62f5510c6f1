"""GPU parity: layer loss tr(dW H dW^T), scale gradient and Adam step against the CPU oracle.

Bar (the benchmark spec): loss, per-row loss, gradient and updated alpha within 1e-5
relative.  The contraction runs on fp32 MFMA with fp32 accumulation; the
oracle is float64 throughout.  Parity is per call on identical inputs: the
oracle is fed the same W, S, H, labels and alpha as the GPU.
"""
import numpy as np
import pytest
import torch

import oracle
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


def make_case(seed, n, m, K, N=None, with_alpha=True):
    W, S = skim_synth.make_ws_small(seed, n, m)
    S = S + np.float32(0.01)
    rng = np.random.default_rng(seed)
    labels = rng.integers(0, K, (n, m)).astype(np.uint8)
    H = skim_synth.make_h_host(3, N or 4 * m, m)
    H = ((H + H.T) / 2).astype(np.float32)
    al = skim_synth.make_alpha(seed, m) if with_alpha else None
    return W, S, labels, H, al


# (m a multiple of 32 from 128 up takes the contraction on the bf16 matrix cores, 256 x 128 tiles: 160 and 416 columns
# leave its last column tile part empty, 70, 260 and 300 rows its last row tile)
@pytest.mark.parametrize("n,m,K", [(1, 16, 2), (37, 48, 4), (130, 144, 8), (257, 272, 16), (128, 512, 16), (300, 1024, 8),
                                   (70, 160, 8), (260, 416, 16)])
@pytest.mark.parametrize("with_alpha", [False, True])
def test_layer_loss_matches_oracle(ctx, n, m, K, with_alpha):
    W, S, labels, H, al = make_case(n + m, n, m, K, with_alpha=with_alpha)
    out = ctx.layer_loss(dev(W), dev(S), dev(H), dev(labels), alpha=None if al is None else dev(al))
    torch.cuda.synchronize()
    c, D = oracle.centroids_from_labels(W, S, labels, al)
    ref = oracle.layer_loss(W, H, labels, c, al)
    assert out["loss"].item() == pytest.approx(ref["loss"], rel=RTOL)
    got = out["row_loss"].cpu().numpy()
    assert np.all(np.abs(got - ref["row_loss"]) <= RTOL * np.abs(ref["row_loss"]) + 1e-9 * ref["loss"] / n)


def test_layer_loss_identity_and_diagonal_hessian(ctx):
    n, m = 64, 256
    W, S, labels, H, al = make_case(5, n, m, 8)
    c, D = oracle.centroids_from_labels(W, S, labels, al)
    dWd = W.astype(np.float64) - al.astype(np.float64)[None, :] * np.take_along_axis(c, labels.astype(np.int64), 1)
    out = ctx.layer_loss(dev(W), dev(S), dev(np.eye(m, dtype=np.float32)), dev(labels), alpha=dev(al))
    torch.cuda.synchronize()
    assert out["loss"].item() == pytest.approx((dWd ** 2).sum(), rel=RTOL)
    h = np.random.default_rng(0).uniform(0.5, 2, m).astype(np.float32)
    out = ctx.layer_loss(dev(W), dev(S), dev(np.diag(h)), dev(labels), alpha=dev(al))
    torch.cuda.synchronize()
    np.testing.assert_allclose(out["row_loss"].cpu().numpy(), (h.astype(np.float64)[None, :] * dWd ** 2).sum(1), rtol=RTOL)


@pytest.mark.parametrize("n,m,K", [(5, 32, 4), (40, 144, 8), (130, 512, 16), (33, 160, 8)])
@pytest.mark.parametrize("t_step", [1, 41])
def test_scale_step_matches_oracle(ctx, gpu_lib, n, m, K, t_step):
    W, S, labels, H, al = make_case(100 + n, n, m, K)
    rng = np.random.default_rng(n)
    m1 = (rng.standard_normal(m) * 1e-3).astype(np.float32) if t_step > 1 else np.zeros(m, np.float32)
    m2 = (rng.uniform(0, 1e-6, m)).astype(np.float32) if t_step > 1 else np.zeros(m, np.float32)
    d_al, d_m1, d_m2 = dev(al), dev(m1), dev(m2)
    out = ctx.scale_step(dev(W), dev(S), dev(H), dev(labels), d_al, d_m1, d_m2, t_step)
    torch.cuda.synchronize()
    ref = oracle.scale_grad(W, S, H, labels, al)
    assert out["loss_before"].item() == pytest.approx(ref["loss"], rel=RTOL)
    g = out["grad"].cpu().numpy().astype(np.float64)
    gscale = np.abs(ref["grad"]).max()
    assert np.all(np.abs(g - ref["grad"]) <= RTOL * np.abs(ref["grad"]) + 1e-6 * gscale)
    # optimiser step on the GPU's own gradient (identical inputs on both sides)
    # the ABI carries the hyper-parameters as float32: the oracle gets the same rounded values
    f32 = lambda x: float(np.float32(x))
    a_ref, m1_ref, m2_ref = oracle.adam_step(al, m1, m2, g, t_step, lr0=f32(0.01), beta1=f32(0.9), beta2=f32(0.999),
                                             eps=f32(1e-8), decay=f32(0.5), decay_every=40)
    np.testing.assert_allclose(d_al.cpu().numpy(), a_ref, rtol=RTOL)
    np.testing.assert_allclose(d_m1.cpu().numpy(), m1_ref, rtol=RTOL, atol=1e-6 * np.abs(m1_ref).max())
    np.testing.assert_allclose(d_m2.cpu().numpy(), m2_ref, rtol=RTOL, atol=1e-6 * np.abs(m2_ref).max())


def test_loss_after_clustering_equals_sdiag_error_when_hessian_is_diagonal(ctx):
    """With H = diag(s_i) the L-full error of a row is its S-diag error; here S is shared by
    all rows so that one H serves every row (ties Sec. 3.3 and 3.4 together end to end)."""
    n, m = 32, 512
    W, _ = skim_synth.make_ws_small(11, n, m)
    s_row = (np.random.default_rng(1).standard_t(3, m) ** 2).astype(np.float32)
    S = np.ascontiguousarray(np.broadcast_to(s_row, (n, m)))
    bits = np.full(n, 3, np.uint8)
    cr = ctx.cluster_rows(dev(W), dev(S), dev(bits))
    out = ctx.layer_loss(dev(W), dev(S), dev(np.diag(s_row)), cr["labels"])
    torch.cuda.synchronize()
    np.testing.assert_allclose(out["row_loss"].cpu().numpy(), cr["err"].cpu().numpy(), rtol=1e-5)


def test_loss_argument_errors(ctx, gpu_lib):
    W, S, labels, H, al = make_case(1, 4, 24, 2)     # m not a multiple of 16
    with pytest.raises(gpu_lib.SkimError):
        ctx.layer_loss(dev(W), dev(S), dev(H), dev(labels))


@pytest.mark.parametrize("n,m,with_alpha,zero_s", [(40, 144, False, 0.0), (130, 512, True, 0.0), (64, 1024, True, 0.0),
                                                   (48, 144, False, 0.9), (48, 272, True, 0.97)])
def test_lfull_error_table_matches_oracle(ctx, n, m, with_alpha, zero_s):
    """Error pre-recording with the layer-wise error: every (row, bit width) entry against the oracle
    (clustering + naive float64 dW H dW^T); rows in which the oracle met a near-tie are excused.  With most
    sensitivities zero some clusters hold members without mass: their centroid is the one the clustering kept."""
    W, S = skim_synth.make_ws_small(21, n, m, zero_s_frac=zero_s)
    H = skim_synth.make_h_host(3, 4 * m, m)
    al = skim_synth.make_alpha(3, m) if with_alpha else None
    ref = oracle.error_table_lfull(W, S, H, alpha=al, count_near=True)
    sd = oracle.error_table(W, S, alpha=al)
    out = ctx.error_table_lfull(dev(W), dev(S), dev(H), alpha=None if al is None else dev(al))
    torch.cuda.synchronize()
    clean = ref["near_rows"] == 0
    assert clean.sum() >= n - 4
    got = out["E_full"].cpu().numpy()
    np.testing.assert_allclose(got[clean], ref["E"][clean], rtol=RTOL)
    np.testing.assert_allclose(out["E"].cpu().numpy()[clean], sd["E"][clean], rtol=RTOL)
    # the S-diag table of the same call equals the plain entry point's, bit for bit
    plain = ctx.error_table(dev(W), dev(S), alpha=None if al is None else dev(al))
    torch.cuda.synchronize()
    assert torch.equal(plain["E"], out["E"]) and torch.equal(plain["upper_all"], out["upper_all"])


def test_train_scale_is_the_composition_of_its_steps_and_tracks_the_oracle(ctx, gpu_lib):
    """skim_train_scale against (a) the same sequence of library calls made one by one: bit-exact; (b) the
    oracle's free-running Alg. 2 on a small, well-conditioned layer: loss trace and alpha within 1e-4 over
    30 steps (per-step parity at 1e-5 is covered by test_scale_step_matches_oracle; a free-running optimiser
    amplifies rounding differences of the fp32 contraction, hence the looser bound here)."""
    n, m = 48, 144
    W, S = skim_synth.make_ws_small(41, n, m)
    S = S + np.float32(0.05)
    H = skim_synth.make_h_host(3, 4 * m, m)
    bits_h = np.full(n, 3, np.uint8)
    Wd, Sd, Hd, bd = dev(W), dev(S), dev(H), dev(bits_h)
    steps = 30
    alpha = torch.ones(m, device="cuda")
    am, av = torch.zeros(m, device="cuda"), torch.zeros(m, device="cuda")
    out = ctx.train_scale(Wd, Sd, Hd, bd, alpha, am, av, steps=steps, outer=2)
    torch.cuda.synchronize()
    # (a) manual composition
    a2 = torch.ones(m, device="cuda")
    m2, v2 = torch.zeros(m, device="cuda"), torch.zeros(m, device="cuda")
    trace = []
    t = 1
    for _ in range(2):
        cr = ctx.cluster_rows(Wd, Sd, bd, alpha=a2)
        for _k in range(steps):
            o = ctx.scale_step(Wd, Sd, Hd, cr["labels"], a2, m2, v2, t, want_grad=False)
            trace.append(o["loss_before"].clone())
            t += 1
    ll = ctx.layer_loss(Wd, Sd, Hd, cr["labels"], alpha=a2)
    trace.append(ll["loss"].clone())
    torch.cuda.synchronize()
    assert torch.equal(alpha, a2) and torch.equal(am, m2) and torch.equal(av, v2)
    assert torch.equal(out["labels"], cr["labels"])
    assert torch.equal(out["loss_trace"], torch.cat([x.reshape(1) for x in trace]))
    c_ref, _ = oracle.centroids_from_labels(W, S, out["labels"].cpu().numpy(), alpha.cpu().numpy())
    np.testing.assert_allclose(out["centroids"].cpu().numpy(), c_ref, rtol=RTOL, atol=1e-12)
    # (b) oracle, free running, one round
    alpha = torch.ones(m, device="cuda")
    am, av = torch.zeros(m, device="cuda"), torch.zeros(m, device="cuda")
    out1 = ctx.train_scale(Wd, Sd, Hd, bd, alpha, am, av, steps=steps)
    torch.cuda.synchronize()
    f32 = lambda x: float(np.float32(x))
    ref = oracle.train_scale(W, S, H, bits_h, np.ones(m, np.float32), steps=steps, lr0=f32(0.01), beta1=f32(0.9),
                             beta2=f32(0.999), eps=f32(1e-8), decay=f32(0.5), decay_every=40)
    np.testing.assert_allclose(out1["loss_trace"].cpu().numpy(), ref["loss_trace"], rtol=1e-4)
    np.testing.assert_allclose(alpha.cpu().numpy(), ref["alpha"], rtol=1e-4)
    assert ref["loss_trace"][-1] < ref["loss_trace"][0]


@pytest.mark.parametrize("N,m", [(40, 12), (300, 130), (1000, 256), (4096, 640),
                                 # wide layers take the kernel with 256 x 256 tiles: a last tile of 8 columns and a
                                 # short first slice of activations; two accumulation chunks; a tile count that is
                                 # no multiple of 8; the fewest activations and the narrowest layer that kernel takes
                                 (200, 3592), (8200, 3840), (128, 4096), (300, 2568)])
def test_hessian_from_activations_matches_oracle(ctx, N, m):
    """H = X^T X / N from bfloat16 activations against the float64 definition: every entry within 1e-5 of the
    entry's natural scale sqrt(H_jj H_ll) (float32 accumulation within a chunk of activations; across chunks
    float64 in the 128 x 128 kernel, float32 -- at most a few dozen additions -- in the 256 x 256 one)."""
    X = np.concatenate(list(skim_synth.make_x(3, N, m)))        # float32 values that are exact in bfloat16
    ref = oracle.hessian_from_activations(X).astype(np.float64)
    Xb = torch.from_numpy(X).cuda().to(torch.bfloat16)
    assert torch.equal(Xb.float().cpu(), torch.from_numpy(X))
    H = ctx.hessian_from_activations(Xb)
    torch.cuda.synchronize()
    got = H.cpu().numpy().astype(np.float64)
    scale = np.sqrt(np.outer(np.diag(ref), np.diag(ref)))
    assert np.all(np.abs(got - ref) <= RTOL * scale), f"max scaled diff {(np.abs(got - ref) / scale).max():.3e}"
    assert torch.equal(H, H.T.contiguous())
