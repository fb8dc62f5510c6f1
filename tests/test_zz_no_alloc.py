"""skim_pack_static, the pack call for callers that cannot allocate: same outputs as skim_pack, bit for bit,
on two calls in a row that share the library's static scratch (the second with a smaller input), and a clear
error beyond the size the scratch holds."""
import numpy as np
import pytest
import torch

import skim_synth

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def pack_both_ways(ctx, n, m, seed, with_alpha, want_dW):
    W, S = skim_synth.make_ws_small(seed, n, m)
    rng = np.random.default_rng(seed)
    bits = rng.integers(1, 5, n).astype(np.uint8)
    al = dev(skim_synth.make_alpha(seed, m)) if with_alpha else None
    Wd, Sd, bd = dev(W), dev(S), dev(bits)
    cr = ctx.cluster_rows(Wd, Sd, bd, alpha=al)
    ref = ctx.pack(Wd, bd, cr["centroids"], cr["upper"], alpha=al, want_dW=want_dW, bits_host=bits)
    torch.cuda.synchronize()
    out = {k: (None if v is None else torch.full_like(v, -1 if v.dtype != torch.float32 else float("nan")))
           for k, v in ref.items()}
    ctx.pack_static(Wd, al, bd, cr["centroids"], cr["upper"], out)
    torch.cuda.synchronize()
    for k, v in ref.items():
        if v is None:
            assert out[k] is None
        else:
            assert torch.equal(out[k], v), f"{k} differs between skim_pack_static and skim_pack (n={n}, m={m})"


def test_static_scratch_pack_matches_pack_on_two_calls_in_a_row(gpu_lib):
    ctx = gpu_lib.Context(0)
    try:
        pack_both_ways(ctx, 300, 1111, 11, with_alpha=True, want_dW=True)
        pack_both_ways(ctx, 37, 257, 12, with_alpha=False, want_dW=False)     # smaller: stale scratch beyond row 37
        pack_both_ways(ctx, 300, 1111, 11, with_alpha=True, want_dW=True)
    finally:
        ctx.close()


def test_static_scratch_pack_needs_no_workspace_and_rejects_oversize(gpu_lib):
    n, m = 64, 320
    W, S = skim_synth.make_ws_small(5, n, m)
    bits = np.full(n, 2, np.uint8)
    Wd, bd = dev(W), dev(bits)
    other = gpu_lib.Context(0)
    ctx = gpu_lib.Context(0)                      # a context that never registers a workspace
    try:
        cr = other.cluster_rows(Wd, dev(S), bd)
        ref = other.pack(Wd, bd, cr["centroids"], cr["upper"], bits_host=bits)
        torch.cuda.synchronize()
        out = {k: (None if v is None else torch.zeros_like(v)) for k, v in ref.items()}
        ctx.pack_static(Wd, None, bd, cr["centroids"], cr["upper"], out)
        torch.cuda.synchronize()
        assert ctx._ws is None
        assert all(v is None or torch.equal(out[k], v) for k, v in ref.items())
        # one row more than the scratch holds: refused before anything is launched
        p = lambda t: t.data_ptr()
        st = ctx.lib.skim_pack_static(ctx.h, p(Wd), None, gpu_lib.PACK_STATIC_MAX_ROWS + 1, m, m, p(bd),
                                      p(cr["centroids"]), p(cr["upper"]), p(out["codes"]), p(out["group_word_offset"]),
                                      p(out["row_perm"]), p(out["codebooks"]), None)
        assert st == -2 and b"static scratch" in ctx.lib.skim_last_error(ctx.h)
    finally:
        ctx.close()
        other.close()
