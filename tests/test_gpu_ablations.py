"""GPU parity for the ablation variants of the correlate and compress stages (the "Correlate"
and "Compress" rows of the paper's two ablation tables; Sec. "Correlation-based Information
Recycling"): fixed K, convergent correlation, average compression, and the pairwise token
correlation gap.  Same bars as the main parity tests."""
import numpy as np
import pytest
import torch

from paper_2411_17686_amd import ficoco as fc
from paper_2411_17686_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = fc.Context(0)
    yield c
    c.close()


def _check_v(cfg, ctx, extra=False, **kw):
    A = cfg.get("A")
    out, _ = P.run_v(cfg, A, ctx=ctx, **kw)
    okw = {k: v for k, v in kw.items() if k not in ("k_max", "staged", "gap")}
    n_keep = kw.get("n_keep", cfg["n_keep"])
    for b in range(cfg["B"]):
        ref = P.oracle_v(cfg, A, b, **okw)
        exact = kw.get("corr_src", fc.C_ATTN) == fc.C_ATTN
        P.compare_image(out, b, ref, cfg["dtype"], cfg["vis_begin"], exact,
                        extra_row=cfg["vis_begin"] + n_keep if extra else None)
        if kw.get("gap"):
            if exact:
                assert np.array_equal(out["gap"][b], ref["gap"])
            else:
                np.testing.assert_allclose(out["gap"][b], ref["gap"], rtol=1e-9, atol=1e-12)
    return out


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("K", [0, 1, 2, 3])
def test_fixed_k_attention(ctx, dtype, K):
    cfg = synth.ficoco_v_single(seed=40 + K, B=2, grid=10, D=72, H=3, centres=5, dtype=dtype, n_keep=37)
    out = _check_v(cfg, ctx, k_mode=fc.K_FIXED, fixed_k=K, gap=True)
    assert np.all(out["cnt"] == K)
    if K == 0:                                   # pruning: the preserved tokens are copies
        X = synth.to_numpy(cfg["X"])
        for b in range(2):
            rows = np.concatenate([[0], 1 + out["keep"][b]])
            assert np.array_equal(out["X_out"][b], X[b][rows])


def test_fixed_k_exact_ties_go_to_the_lower_position(ctx):
    """Duplicated query rows make correlations tie exactly: of equal values only the lowest
    positions are taken, exactly K targets per discarded token."""
    cfg = synth.ficoco_v_single(seed=44, B=2, grid=8, D=32, H=4, centres=3, dtype="bf16", n_keep=30)
    A = cfg["A"].clone()
    for (src, dst) in [(5, 9), (5, 17), (20, 21), (33, 40), (33, 41)]:
        A[:, :, dst, :] = A[:, :, src, :]
    cfg["A"] = A
    for K in (1, 2, 3):
        out = _check_v(cfg, ctx, k_mode=fc.K_FIXED, fixed_k=K, window=0)
        assert np.all(out["cnt"] == K)
    cfg["A"] = torch.full_like(A, 1.0 / 65)      # every correlation ties: targets 0 .. K-1
    out = _check_v(cfg, ctx, k_mode=fc.K_FIXED, fixed_k=3, window=0)
    assert np.all(out["tgt"][:, :, :3] == np.arange(3))


def test_fixed_k_larger_than_register_lists(ctx):
    """K above the 8 order statistics kept in registers: the dense-row path."""
    cfg = synth.ficoco_v_single(seed=45, B=2, grid=9, D=40, H=2, centres=4, dtype="bf16", n_keep=40)
    out = _check_v(cfg, ctx, k_mode=fc.K_FIXED, fixed_k=12, k_max=16)
    assert np.all(out["cnt"] == 12)
    _check_v(cfg, ctx, k_mode=fc.K_FIXED, fixed_k=12, k_max=16, corr_src=fc.C_COSINE)


def test_fixed_k_cosine_and_l(ctx):
    cfg = synth.ficoco_v_video(seed=46, B=2, frames=3, grid=8, D=96, H=4, centres=6, n_keep=40)
    for K in (1, 2):
        _check_v(cfg, ctx, red_src=fc.R_VECTOR, sem_src=fc.G_VECTOR, corr_src=fc.C_COSINE,
                 k_mode=fc.K_FIXED, fixed_k=K, gap=True)
    for with_vv in (False, True):
        cfg = synth.ficoco_l_decoder(seed=47, B=2, n_sys=5, N=100, M=12, D=128, H=4, centres=8,
                                     n_keep=30, with_vv=with_vv)
        red, cor = (fc.R_ATTN_RECV, fc.C_ATTN) if with_vv else (fc.R_SIM_MEAN, fc.C_COSINE)
        for kw in (dict(k_mode=fc.K_FIXED, fixed_k=2), dict(k_mode=fc.K_FIXED, fixed_k=0),
                   dict(compress_mode=fc.COMPRESS_AVERAGE), dict(k_mode=fc.K_CONVERGENT)):
            out, _ = P.run_l(cfg, red, cor, ctx=ctx, gap=True, **kw)
            for b in range(2):
                ref = P.oracle_l(cfg, b, red, cor, **kw)
                extra = cfg["vis_begin"] + cfg["n_keep"] if kw.get("k_mode") == fc.K_CONVERGENT else None
                P.compare_image(out, b, ref, "bf16", cfg["vis_begin"], False, extra_row=extra)
                np.testing.assert_allclose(out["gap"][b], ref["gap"], rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_average_compression(ctx, dtype):
    cfg = synth.ficoco_v_single(seed=48, B=2, grid=10, D=100, H=3, centres=5, dtype=dtype, n_keep=30)
    _check_v(cfg, ctx, compress_mode=fc.COMPRESS_AVERAGE, eps=0.9, k_max=16)
    _check_v(cfg, ctx, compress_mode=fc.COMPRESS_AVERAGE, k_mode=fc.K_FIXED, fixed_k=2)
    # the inverted-list path of the merge (more than 1024 discarded tokens)
    cfg = synth.ficoco_v_multicrop(seed=49, B=1, crops=3, grid=24, D=64, H=2, centres=20, n_keep=300)
    _check_v(cfg, ctx, compress_mode=fc.COMPRESS_AVERAGE)


@pytest.mark.parametrize("dtype,D", [("f32", 100), ("bf16", 1030)])
def test_convergent_token(ctx, dtype, D):
    cfg = synth.ficoco_v_single(seed=50, B=2, grid=9, D=D, H=2, centres=5, dtype=dtype, n_keep=33)
    out = _check_v(cfg, ctx, extra=True, k_mode=fc.K_CONVERGENT)
    assert out["X_out"].shape[1] == 1 + 33 + 1 and np.all(out["cnt"] == 0)
    # zero discards: no extra token, identity
    out = _check_v(cfg, ctx, k_mode=fc.K_CONVERGENT, n_keep=81)
    assert np.array_equal(out["X_out"], synth.to_numpy(cfg["X"]))
    # many discarded tokens (inverted-list merge mode), several feature spans
    cfg = synth.ficoco_v_multicrop(seed=51, B=1, crops=3, grid=24, D=64, H=2, centres=20, n_keep=300)
    out = _check_v(cfg, ctx, extra=True, k_mode=fc.K_CONVERGENT)
    assert out["X_out"].shape[1] == 1 + 300 + 1


def test_ablation_argument_errors(ctx):
    cfg = synth.ficoco_v_single(seed=52, B=1, grid=6, D=32, H=2, centres=3, dtype="bf16", n_keep=20)
    with pytest.raises(fc.FicocoError):
        P.run_v(cfg, cfg["A"], ctx=ctx, k_mode=fc.K_FIXED, fixed_k=9, k_max=8)     # above k_max
    with pytest.raises(fc.FicocoError):
        P.run_v(cfg, cfg["A"], ctx=ctx, k_mode=7)
    with pytest.raises(fc.FicocoError):
        P.run_v(cfg, cfg["A"], ctx=ctx, compress_mode=5)
