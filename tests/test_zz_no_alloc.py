"""The allocation-free entry point ficoco_v_step_static (workspace = the library's static device
array) against ficoco_v_step (caller workspace): every output must be identical, on two calls
in a row, the second on a smaller problem (the array then still holds the first call's data).
One image per call is also compared with the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2411_17686_amd import ficoco as fc
from paper_2411_17686_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu


def _problem(cfg):
    Xd, Ad = cfg["X"].to("cuda"), cfg["A"].to("cuda")
    p = fc.make_problem(Xd, variant=fc.VARIANT_V, vis_begin=cfg["vis_begin"], N=cfg["N"], n_keep=cfg["n_keep"],
                        A=Ad, cls_index=cfg["cls_index"], grid=cfg["grid"], window=cfg["window"],
                        penalty_coef=cfg["coef"], w_score=cfg["lam"], eps=cfg["eps"], k_max=8, H=cfg["H"])
    return p, (Xd, Ad)


def test_static_scratch_step_equals_workspace_step():
    ctx = fc.Context(0)
    cases = [synth.ficoco_v_single(seed=21, B=4, grid=24, D=256, H=4, centres=16, dtype="bf16", n_keep=384),
             synth.ficoco_v_single(seed=22, B=2, grid=12, D=136, H=3, centres=8, dtype="f32", n_keep=48)]
    for cfg in cases:
        p, keep_alive = _problem(cfg)
        assert fc.workspace_bytes(p) <= fc.STATIC_SCRATCH_BYTES
        want_buf = fc.Buffers(p, "cuda", keep_alive[0].dtype)
        fc.ficoco_v_step(ctx, p, want_buf)
        want = P.gpu_outputs(want_buf)
        got_buf = fc.Buffers(p, "cuda", keep_alive[0].dtype)
        got_buf.ws = None                                   # the static entry point takes no workspace
        fc.ficoco_v_step_static(ctx, p, got_buf)
        got = P.gpu_outputs(got_buf)
        for k in ("X_out", "pos_out", "keep", "discard", "cnt", "tgt", "alpha", "scores", "overflow"):
            assert np.array_equal(got[k], want[k]), k
        ref = P.oracle_v(cfg, cfg["A"], 0)
        P.compare_image(got, 0, ref, cfg["dtype"], cfg["vis_begin"], True)
        del keep_alive
    ctx.close()


def test_static_scratch_rejects_a_step_that_does_not_fit():
    ctx = fc.Context(0)
    cfg = synth.ficoco_v_single(seed=23, B=1, grid=4, D=8, H=1, centres=2, dtype="bf16", n_keep=8)
    p, keep_alive = _problem(cfg)
    buf = fc.Buffers(p, "cuda", keep_alive[0].dtype)
    # The same pointers described as 200 images of 576 patches: the step would need about 80 MB.  The
    # call must be refused on the host, before any kernel could touch memory that is not there.
    p.B, p.N, p.n_tot, p.n_keep, p.a_nq, p.a_nk = 200, 576, 577, 384, 577, 577
    p.grid_h = p.grid_w = 24
    p.a_stride_q, p.a_stride_h, p.a_stride_b = 577, 577 * 577, 577 * 577
    p.x_stride_n, p.x_stride_b = p.D, 577 * p.D
    assert fc.workspace_bytes(p) > fc.STATIC_SCRATCH_BYTES
    with pytest.raises(fc.FicocoError) as e:
        fc.ficoco_v_step_static(ctx, p, buf)
    assert e.value.code == fc.ENOMEM
    torch.cuda.synchronize()
    del keep_alive
    ctx.close()
