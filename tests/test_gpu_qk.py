"""The step fed with projected queries and keys instead of the attention maps (Sec.
"Self-Attention", A = Softmax(Q K^T / sqrt(D))): the library forms the per-head softmax on the
matrix cores in single precision and never stores [B,H,n,n]; the oracle forms it in float64.

Bar.  Scores and map entries agree to about 1e-6, not to the last bit, so the comparison is the
margin rule: every top-K decision and every threshold decision whose relative margin (from the
oracle's float64 values) exceeds 64 * 2^-24 must be identical; where all decisions of an image are
identical, weights and merged tokens must agree within the token tolerance (bfloat16: 2e-2
relative / 1e-2 absolute; float32: 1e-5 of the row's largest magnitude)."""
import sys

import numpy as np
import pytest
import torch

from oracle import ficoco_oracle as O
from paper_2411_17686_amd import ficoco as fc
from paper_2411_17686_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def draw_qk(seed, B, H, n, d, sigma):
    """Queries and keys whose logits q.k / sqrt(d) are about N(0, sigma^2), as bfloat16."""
    g = torch.Generator().manual_seed(seed)
    Q = (torch.randn(B, H, n, d, generator=g) * sigma ** 0.5).to(torch.bfloat16)
    K = (torch.randn(B, H, n, d, generator=g) * sigma ** 0.5).to(torch.bfloat16)
    return Q, K


def run_qk(ctx, cfg, Q, K, **kw):
    Xd, Qd, Kd = cfg["X"].to("cuda"), Q.to("cuda"), K.to("cuda")
    p = fc.make_problem(Xd, variant=fc.VARIANT_V, vis_begin=cfg["vis_begin"], N=cfg["N"], n_keep=cfg["n_keep"],
                        cls_index=cfg["cls_index"], grid=cfg["grid"], window=cfg["window"], penalty_coef=cfg["coef"],
                        w_score=cfg["lam"], eps=cfg["eps"], Q=Qd, K=Kd, qk_begin=0, **kw)
    buf = fc.Buffers(p, "cuda", Xd.dtype)
    fc.ficoco_v_step(ctx, p, buf)
    out = P.gpu_outputs(buf)
    del Xd, Qd, Kd
    return out


def compare_under_margin_rule(out, b, ref, dtype, vis_begin):
    """Returns True when every decision of the image agreed (then the values were compared too)."""
    scale = float(np.max(np.abs(ref["scores"])))
    assert np.all(np.abs(out["scores"][b] - ref["scores"]) <= 8e-6 * scale), "scores beyond single-precision accuracy"
    same_sets = np.array_equal(out["discard"][b], ref["S"])
    if not same_sets:
        # only decisions inside the margin may differ: checked token by token
        P.margin_audit(dict(out, cnt=np.zeros_like(out["cnt"])), b, dict(ref, tau=None))
        return False
    P.margin_audit(out, b, ref)
    same_J = all(out["cnt"][b, a] == len(J) and np.array_equal(out["tgt"][b, a, :len(J)], J)
                 for a, J in enumerate(ref["J"]))
    if not same_J:
        return False
    for a, J in enumerate(ref["J"]):
        np.testing.assert_allclose(out["alpha"][b, a, :len(J)], ref["alpha"][a], rtol=2e-5)
    got, want = O.widen(out["X_out"][b]), ref["X_out"]
    err = np.abs(got - want)
    if dtype == "f32":
        assert np.all(err <= 1e-5 * np.max(np.abs(want), axis=1, keepdims=True))
    else:
        assert np.all(err <= 2e-2 * np.abs(want) + 1e-2)
    if ref["pos_out"] is not None:
        assert np.array_equal(out["pos_out"][b], ref["pos_out"])
    return True


@pytest.fixture(scope="module")
def ctx():
    c = fc.Context(0)
    yield c
    c.close()


def _case(ctx, seed, B, grid, D, H, d, dtype, n_keep, sigma):
    cfg = synth.ficoco_v_single(seed=seed, B=B, grid=grid, D=D, H=1, centres=8, dtype=dtype, n_keep=n_keep)
    Q, K = draw_qk(seed + 1, B, H, cfg["N"] + 1, d, sigma)
    out = run_qk(ctx, cfg, Q, K)
    full = 0
    for b in range(B):
        ref = O.v_step_qk(O.widen(synth.to_numpy(cfg["X"][b])), O.widen(synth.to_numpy(Q[b])), O.widen(synth.to_numpy(K[b])),
                          float(d) ** -0.5, cls_index=0, vis_begin=1, N=cfg["N"], n_keep=n_keep, lam=cfg["lam"],
                          eps=cfg["eps"], grid=cfg["grid"], window=2, coef=2.0)
        full += compare_under_margin_rule(out, b, ref, dtype, 1)
    return full


def test_config0_shape_from_queries_and_keys(ctx):
    full = _case(ctx, 40, 1, 24, 1024, 16, 64, "f32", 192, 1.0)
    say("config 0 shape from Q, K: %d of 1 images with every decision identical" % full)


def test_config1_shape_from_queries_and_keys(ctx):
    full = _case(ctx, 41, 16, 24, 1024, 16, 64, "bf16", 384, 1.5)
    say("config 1 shape from Q, K: %d of 16 images with every decision identical" % full)
    assert full >= 12          # in-margin decisions are rare


@pytest.mark.parametrize("seed,grid,H,d,n_keep", [(1, 7, 3, 32, 20), (2, 16, 5, 32, 100), (3, 19, 2, 128, 301), (4, 25, 4, 64, 625),
                                                  (5, 5, 1, 64, 1)])
def test_small_and_ragged_shapes(ctx, seed, grid, H, d, n_keep):
    full = _case(ctx, 50 + seed, 2, grid, 72, H, d, ["f32", "bf16"][seed % 2], n_keep, 1.0)
    assert full >= 1


def test_long_sequence_at_full_width_from_queries_and_keys(ctx):
    """2304 patches + [CLS], 16 heads of 64, D = 1024, 640 preserved (the size class of BASELINE
    config 2): four key blocks, the last of 385 keys."""
    full = _case(ctx, 42, 2, 48, 1024, 16, 64, "bf16", 640, 1.0)
    say("2304-patch shape from Q, K: %d of 2 images with every decision identical" % full)


@pytest.mark.parametrize("seed,grid,H,d,n_keep", [(1, 27, 3, 64, 300), (2, 36, 2, 32, 500), (3, 31, 5, 128, 700),
                                                  (4, 40, 1, 64, 1000)])
def test_sequences_longer_than_one_key_block(ctx, seed, grid, H, d, n_keep):
    """More than 640 keys: the keys are taken in blocks of 640 in two sweeps (normalisers of every
    head first, then the probabilities block by block).  730 keys: a second block of 90; 1297: a
    third block of 17, most of whose wavefronts hold no key; 962 and 1601 with one to five heads."""
    full = _case(ctx, 70 + seed, 2, grid, 72, H, d, ["f32", "bf16"][seed % 2], n_keep, 1.0)
    assert full >= 1


def _case_l(ctx, seed, B, n_sys, N, M, D, H, d, n_keep, red, corr, sigma=1.0, staged=False):
    """FiCoCo-L fed the decoder layer's queries and keys (causal maps; the text tokens follow the
    visual span) against the oracle's float64 evaluation, under the margin rule."""
    cfg = synth.ficoco_l_decoder(seed=seed, B=B, n_sys=n_sys, N=N, M=M, D=D, H=1, centres=8, n_keep=n_keep, with_vv=False)
    n_tot = n_sys + N + M
    Q, K = draw_qk(seed + 1, B, H, n_tot, d, sigma)
    Xd, Qd, Kd = cfg["X"].to("cuda"), Q.to("cuda"), K.to("cuda")
    p = fc.make_problem(Xd, variant=fc.VARIANT_L, vis_begin=n_sys, N=N, n_keep=n_keep, w_score=cfg["beta"],
                        gamma=cfg["gamma"], eps=cfg["eps"], red_src=red, sem_src=fc.G_TEXT_ATTN, corr_src=corr,
                        window=0, Q=Qd, K=Kd, qk_begin=0, M=M)
    buf = fc.Buffers(p, "cuda", Xd.dtype)
    if staged:
        fc.ficoco_score(ctx, p, buf)
        fc.ficoco_filter(ctx, p, buf)
        fc.ficoco_correlate(ctx, p, buf)
        fc.ficoco_compress(ctx, p, buf)
    else:
        fc.ficoco_l_step(ctx, p, buf)
    out = P.gpu_outputs(buf)
    del Xd, Qd, Kd
    full = 0
    names = {fc.R_ATTN_RECV: "attn", fc.R_SIM_MEAN: "sim_mean", fc.C_ATTN: "attn", fc.C_COSINE: "cosine"}
    for b in range(B):
        ref = O.l_step_qk(O.widen(synth.to_numpy(cfg["X"][b])), O.widen(synth.to_numpy(Q[b])), O.widen(synth.to_numpy(K[b])),
                          float(d) ** -0.5, vis_begin=n_sys, N=N, M=M, n_keep=n_keep, beta=cfg["beta"], gamma=cfg["gamma"],
                          eps=cfg["eps"], red_src=names[red], corr_src="attn" if corr == fc.C_ATTN else "cosine")
        full += compare_under_margin_rule(out, b, ref, cfg["dtype"], n_sys)
    return full


@pytest.mark.parametrize("red,corr", [(fc.R_ATTN_RECV, fc.C_ATTN), (fc.R_SIM_MEAN, fc.C_COSINE), (fc.R_ATTN_RECV, fc.C_COSINE)])
@pytest.mark.parametrize("shape", [(3, 77, 9, 72, 3, 32, 31), (35, 576, 64, 128, 4, 64, 144), (5, 1300, 40, 72, 2, 128, 700),
                                   (0, 100, 1, 64, 1, 64, 50)])
def test_decoder_step_from_queries_and_keys(ctx, shape, red, corr):
    """89, 675 (the decoder shape of BASELINE config 3: two key blocks), 1345 and 101 positions; with
    the visual-to-visual terms (tiles over the visual and the text queries) and without (text queries
    alone); 1 to 64 text queries."""
    n_sys, N, M, D, H, d, n_keep = shape
    full = _case_l(ctx, 80 + N % 50, 2, n_sys, N, M, D, H, d, n_keep, red, corr)
    assert full >= 1


@pytest.mark.parametrize("red,corr", [(fc.R_ATTN_RECV, fc.C_ATTN), (fc.R_SIM_MEAN, fc.C_COSINE)])
def test_decoder_stages_from_queries_and_keys(ctx, red, corr):
    """The same through the staged entry points (score, filter, correlate, compress one call each)."""
    assert _case_l(ctx, 91, 2, 4, 130, 33, 72, 6, 64, 60, red, corr, staged=True) >= 1


def test_unsupported_shapes_are_refused(ctx):
    cfg = synth.ficoco_v_single(seed=9, B=1, grid=4, D=8, H=1, centres=2, dtype="bf16", n_keep=8)
    Xd = cfg["X"].to("cuda")
    for n, d in ((17, 24), (17, 16), (17, 256)):
        Q = torch.zeros(1, 2, n, d, dtype=torch.bfloat16, device="cuda")
        p = fc.make_problem(Xd, variant=fc.VARIANT_V, vis_begin=1, N=16, n_keep=8, cls_index=0, grid=(1, 4, 4), window=2,
                            Q=Q, K=Q.clone())
        with pytest.raises(fc.FicocoError) as e:
            fc.workspace_bytes(p)
        assert e.value.code == fc.EUNSUPPORTED
    # beyond 640 rows the normalisers of all heads are kept on chip: at most 64 heads
    cfg = synth.ficoco_v_single(seed=9, B=1, grid=26, D=8, H=1, centres=2, dtype="bf16", n_keep=8)
    Xd = cfg["X"].to("cuda")
    Q = torch.zeros(1, 65, 677, 32, dtype=torch.bfloat16, device="cuda")
    p = fc.make_problem(Xd, variant=fc.VARIANT_V, vis_begin=1, N=676, n_keep=8, cls_index=0, grid=(1, 26, 26), window=2,
                        Q=Q, K=Q.clone())
    with pytest.raises(fc.FicocoError) as e:
        fc.workspace_bytes(p)
    assert e.value.code == fc.EUNSUPPORTED
