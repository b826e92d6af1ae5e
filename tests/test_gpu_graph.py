"""The fused step under HIP graph capture: every call of the library is a plain sequence of
kernel launches on the caller's stream (no allocation, no synchronisation, no memset node), so a
caller may capture it.  The graph is replayed several times with fresh inputs written into the same
buffers, with eager work and synchronisations between the replays, and every replay is compared
with the eager result of the same inputs."""
import numpy as np
import pytest
import torch

from paper_2411_17686_amd import ficoco as fc
from paper_2411_17686_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["attn", "cosine"])
def test_v_step_graph_replays_match_eager(mode):
    ctx = fc.Context(0)
    cfgs = [synth.ficoco_v_single(seed=80 + k, B=2, grid=12, D=160, H=4, centres=6, dtype="bf16", n_keep=60)
            for k in range(3)]
    Xd, Ad = P.dev(cfgs[0]["X"]).clone(), P.dev(cfgs[0]["A"]).clone()
    c = cfgs[0]
    kw = dict(corr_src=fc.C_COSINE) if mode == "cosine" else {}
    p = fc.make_problem(Xd, variant=fc.VARIANT_V, vis_begin=1, N=144, n_keep=60, A=Ad, cls_index=0,
                        grid=c["grid"], window=c["window"], penalty_coef=c["coef"], w_score=c["lam"], eps=c["eps"], **kw)
    eager_buf = fc.Buffers(p, "cuda", Xd.dtype)
    graph_buf = fc.Buffers(p, "cuda", Xd.dtype)
    side = torch.cuda.Stream()
    fc.ficoco_v_step(ctx, p, graph_buf)               # warm-up outside the capture (function attributes, module load)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        fc.ficoco_v_step(ctx, p, graph_buf)
    for k in (1, 2, 0, 1):
        Xd.copy_(P.dev(cfgs[k]["X"])); Ad.copy_(P.dev(cfgs[k]["A"]))
        torch.cuda.synchronize()
        fc.ficoco_v_step(ctx, p, eager_buf)            # eager work between the replays
        want = P.gpu_outputs(eager_buf)
        for name in ("X_out", "keep_idx", "discard_idx", "edge_cnt", "scores", "overflow", "pos_out"):
            getattr(graph_buf, name).zero_()
        torch.cuda.synchronize()
        g.replay()
        got = P.gpu_outputs(graph_buf)
        for name in ("X_out", "keep", "discard", "cnt", "scores", "overflow", "pos_out"):
            assert np.array_equal(got[name], want[name]), (k, name)
        for b in range(2):                             # edge lists: only the filled part is defined
            for a in range(got["cnt"].shape[1]):
                n = got["cnt"][b, a]
                assert np.array_equal(got["tgt"][b, a, :n], want["tgt"][b, a, :n])
                assert np.array_equal(got["alpha"][b, a, :n], want["alpha"][b, a, :n])
        ref = P.oracle_v(cfgs[k], cfgs[k]["A"], 0, **kw)
        P.compare_image(got, 0, ref, "bf16", 1, mode == "attn")
    ctx.close()
