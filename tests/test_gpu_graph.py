"""The clustering call under a HIP graph.  The row sort hands its units of work out from a counter that the last
workgroup of a launch leaves at zero; a captured launch must find it so on every replay, also with eager calls of
the same context in between.  Replays are checked against the eager result, bit for bit (same kernels, same inputs:
the results do not depend on which workgroup sorted a row)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_error_table_replays_from_a_captured_graph(gpu_lib):
    stream = torch.cuda.Stream()
    ctx = gpu_lib.Context(0, stream=stream)
    try:
        # more rows than workgroups resident at once (two per compute unit at this length): most units are claimed
        n, m = 1500, 4096
        rng = np.random.default_rng(812)
        W = (rng.standard_normal((n, m)) * 0.02).astype(np.float32)
        S = (rng.standard_normal((n, m)) ** 2).astype(np.float32)
        W2 = (rng.standard_normal((n, m)) * 0.05).astype(np.float32)
        with torch.cuda.stream(stream):
            Wd, Sd, W2d = torch.from_numpy(W).cuda(), torch.from_numpy(S).cuda(), torch.from_numpy(W2).cuda()
            eager = ctx.error_table(Wd, Sd)
            out = {k: torch.empty_like(v) for k, v in eager.items()}
            other = ctx.error_table(W2d, Sd)
        stream.synchronize()
        ref = {k: v.clone() for k, v in eager.items()}
        ref_other = {k: v.clone() for k, v in other.items()}
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            ctx.error_table(Wd, Sd, out=out)
        for rep in range(4):
            with torch.cuda.stream(stream):
                for v in out.values():
                    v.zero_()
                ctx.error_table(W2d, Sd, out=other)      # eager work of the same context between the replays
                graph.replay()
            stream.synchronize()
            for k in ref:
                assert torch.equal(out[k], ref[k]), f"replay {rep}: {k} differs from the eager call"
                assert torch.equal(other[k], ref_other[k]), f"replay {rep}: eager {k} changed"
    finally:
        ctx.close()
