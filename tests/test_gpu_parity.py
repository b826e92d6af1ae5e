"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded
inputs.  Sizes here are ones the oracle finishes in seconds while spanning several tiles
and ragged tails; the full BASELINE configurations are in test_gpu_configs.py."""
import numpy as np
import pytest
import torch

from oracle import ficoco_oracle as O
from paper_2411_17686_amd import ficoco as fc
from paper_2411_17686_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = fc.Context(0)
    yield c
    c.close()


def _check_v(cfg, ctx, **kw):
    A = cfg.get("A")
    out, _ = P.run_v(cfg, A, ctx=ctx, **kw)
    okw = {k: v for k, v in kw.items() if k not in ("k_max", "staged")}
    worst = 0.0
    for b in range(cfg["B"]):
        ref = P.oracle_v(cfg, A, b, **okw)
        exact = kw.get("corr_src", fc.C_ATTN) == fc.C_ATTN
        worst = max(worst, P.compare_image(out, b, ref, cfg["dtype"], cfg["vis_begin"], exact))
    return out, worst


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("grid,D,H,B,keep", [(8, 64, 4, 2, 20), (12, 200, 3, 3, 100), (5, 37, 2, 2, 7),
                                            (24, 128, 16, 2, 192)])
def test_v_step_small(ctx, dtype, grid, D, H, B, keep):
    cfg = synth.ficoco_v_single(seed=10 + grid, B=B, grid=grid, D=D, H=H, centres=6, dtype=dtype,
                                n_keep=keep)
    _check_v(cfg, ctx)


def test_v_step_staged_equals_fused(ctx):
    cfg = synth.ficoco_v_single(seed=3, B=2, grid=10, D=96, H=4, centres=5, dtype="bf16", n_keep=40)
    fused, _ = P.run_v(cfg, cfg["A"], ctx=ctx)
    staged, _ = P.run_v(cfg, cfg["A"], ctx=ctx, staged=True)
    for k in fused:
        assert np.array_equal(fused[k], staged[k]), k
    again, _ = P.run_v(cfg, cfg["A"], ctx=ctx)            # run-twice determinism
    for k in fused:
        assert np.array_equal(fused[k], again[k]), k


def test_v_step_zero_discards_is_identity(ctx):
    cfg = synth.ficoco_v_single(seed=4, B=2, grid=6, D=40, H=2, centres=4, dtype="bf16", n_keep=36)
    out, _ = P.run_v(cfg, cfg["A"], ctx=ctx)
    assert np.array_equal(out["X_out"], synth.to_numpy(cfg["X"]))
    assert np.array_equal(out["keep"], np.tile(np.arange(36, dtype=np.int32), (2, 1)))


@pytest.mark.parametrize("eps,k_max", [(1.0, 8), (0.0, 64), (0.0, 100), (0.5, 80), (0.9, 16)])
def test_v_step_quantile_range(ctx, eps, k_max):
    """eps = 1 (arg-max), eps = 0 (every target) and mid-range quantiles: the dense
    selection path and edge lists longer than a wavefront."""
    cfg = synth.ficoco_v_single(seed=5, B=2, grid=10, D=48, H=3, centres=5, dtype="f32", n_keep=64)
    if eps == 0.0 and k_max == 100:
        cfg = synth.ficoco_v_single(seed=5, B=2, grid=12, D=48, H=3, centres=5, dtype="f32", n_keep=100)
    _check_v(cfg, ctx, eps=eps, k_max=k_max)


def test_v_step_overflow_flag(ctx):
    cfg = synth.ficoco_v_single(seed=6, B=2, grid=8, D=32, H=2, centres=4, dtype="f32", n_keep=30)
    out, _ = P.run_v(cfg, cfg["A"], ctx=ctx, eps=0.5, k_max=4)
    assert np.all(out["overflow"] == 1)
    assert np.all(out["cnt"] == 4)


def test_v_step_exact_ties(ctx):
    """Duplicated attention columns and query rows: scores tie exactly, correlations tie
    exactly; the lower index is discarded first and tied targets are all selected."""
    cfg = synth.ficoco_v_single(seed=7, B=2, grid=8, D=32, H=4, centres=3, dtype="bf16", n_keep=30)
    A = cfg["A"].clone()
    for (src, dst) in [(5, 9), (5, 17), (20, 21), (33, 40)]:
        A[:, :, :, dst] = A[:, :, :, src]
        A[:, :, dst, :] = A[:, :, src, :]
    cfg["A"] = A
    _check_v(cfg, ctx, window=0)
    _check_v(cfg, ctx)
    # all scores equal: uniform attention (every correlation ties too: J_i = all 30 targets)
    cfg["A"] = torch.full_like(A, 1.0 / 65)
    out, _ = _check_v(cfg, ctx, window=0, k_max=32)
    assert np.array_equal(out["discard"][0], np.arange(34))


def test_v_step_with_positions_and_padding(ctx):
    """Second-step situation: fewer tokens than grid cells, explicit pos."""
    cfg = synth.ficoco_v_single(seed=8, B=3, grid=7, D=64, H=2, centres=4, dtype="bf16", n_keep=20)
    cfg["grid"] = (1, 9, 9)
    g = torch.Generator().manual_seed(0)
    pos = torch.stack([torch.randperm(81, generator=g)[:49].sort().values for _ in range(3)]).to(torch.int32)
    out, _ = P.run_v(cfg, cfg["A"], ctx=ctx, pos=pos)
    for b in range(3):
        ref = P.oracle_v(cfg, cfg["A"], b, pos=pos)
        P.compare_image(out, b, ref, "bf16", 1, True)


def test_v_step_multigrid_wide(ctx):
    """More key columns than one strip of the reduction kernel (N = 3 * 28 * 28 = 2352)."""
    cfg = synth.ficoco_v_multicrop(seed=9, B=1, crops=3, grid=28, D=64, H=2, centres=20, n_keep=500)
    _check_v(cfg, ctx)


def test_v_step_vector_and_cosine(ctx):
    cfg = synth.ficoco_v_video(seed=11, B=2, frames=3, grid=8, D=96, H=4, centres=6, n_keep=40)
    _check_v(cfg, ctx, red_src=fc.R_VECTOR, sem_src=fc.G_VECTOR, corr_src=fc.C_COSINE)


def test_v_step_eq_token_and_sim_mean(ctx):
    cfg = synth.ficoco_v_single(seed=12, B=2, grid=9, D=72, H=2, centres=5, dtype="bf16", n_keep=30)
    _check_v(cfg, ctx, sem_src=fc.G_EQ_TOKEN)
    _check_v(cfg, ctx, red_src=fc.R_SIM_MEAN, sem_src=fc.G_EQ_TOKEN, corr_src=fc.C_COSINE)
    cfg = synth.ficoco_v_single(seed=13, B=1, grid=6, D=50, H=2, centres=5, dtype="f32", n_keep=12)
    g = torch.Generator().manual_seed(1)
    F = torch.randn(1, 36, 24, generator=g)
    _check_v(cfg, ctx, sem_src=fc.G_EQ_TOKEN, corr_src=fc.C_COSINE, F=F)


@pytest.mark.parametrize("with_vv", [False, True])
def test_l_step_small(ctx, with_vv):
    cfg = synth.ficoco_l_decoder(seed=14, B=2, n_sys=5, N=100, M=12, D=128, H=4, centres=8,
                                 n_keep=30, with_vv=with_vv)
    red, cor = (fc.R_ATTN_RECV, fc.C_ATTN) if with_vv else (fc.R_SIM_MEAN, fc.C_COSINE)
    out, _ = P.run_l(cfg, red, cor, ctx=ctx)
    for b in range(2):
        ref = P.oracle_l(cfg, b, red, cor)
        P.compare_image(out, b, ref, "bf16", cfg["vis_begin"], False)
    staged, _ = P.run_l(cfg, red, cor, ctx=ctx, staged=True)
    for k in out:
        assert np.array_equal(out[k], staged[k]), k


def test_error_paths(ctx):
    cfg = synth.ficoco_v_single(seed=1, B=1, grid=4, D=16, H=2, centres=2, dtype="f32", n_keep=8)
    Xd, Ad = cfg["X"].cuda(), cfg["A"].cuda()
    p = fc.make_problem(Xd, variant=fc.VARIANT_V, vis_begin=1, N=16, n_keep=8, A=Ad, cls_index=0,
                        grid=(1, 4, 4), window=2)
    buf = fc.Buffers(p, "cuda", Xd.dtype)
    with pytest.raises(fc.FicocoError) as e:
        fc.ficoco_l_step(ctx, p, buf)
    assert e.value.code == fc.EINVAL
    buf.ws_bytes = 16
    with pytest.raises(fc.FicocoError) as e:
        fc.ficoco_v_step(ctx, p, buf)
    assert e.value.code == fc.ENOMEM


def _sink_attention(n, j_star, c0, dtype):
    """Map in which every query but j_star puts nearly all of its mass on key c0, and j_star
    attends uniformly: for every key i != c0 the strongest query is j_star, so every
    discarded token names the same target."""
    eps = 1e-4
    P = torch.full((n, n), eps)
    P[:, c0] = 1.0 - eps * (n - 1)
    P[j_star, :] = 1.0 / n
    return P[None, None].to(torch.bfloat16 if dtype == "bf16" else torch.float32).contiguous()


@pytest.mark.parametrize("N,n_keep,D", [(100, 30, 40), (1300, 150, 16)])
def test_v_step_many_sources_on_one_target(ctx, N, n_keep, D):
    """More sources on one preserved token than the merge kernel lists in LDS: 69 via the
    scanning path (N = 100) and > 1000 via the inverted-list path (N = 1300)."""
    cfg = synth.ficoco_v_single(seed=21, B=1, grid=10, D=D, H=1, centres=4, dtype="f32", n_keep=n_keep)
    g = torch.Generator().manual_seed(5)
    cfg["X"] = torch.randn(1, N + 1, D, generator=g)
    cfg["A"] = _sink_attention(N + 1, N, 1, "f32")      # j_star = last token (kept: ties discard low indices)
    cfg["grid"] = (1, 1, N)
    out, _ = P.run_v(cfg, cfg["A"], ctx=ctx, window=0)
    ref = P.oracle_v(cfg, cfg["A"], 0, window=0)
    P.compare_image(out, 0, ref, "f32", 1, True)
    hits = sum(1 for j in ref["J"] if len(j) == 1 and j[0] == n_keep - 1)
    assert hits > 64


def test_staged_equals_fused_cosine_and_l(ctx):
    cfg = synth.ficoco_v_video(seed=31, B=2, frames=2, grid=8, D=64, H=2, centres=5, n_keep=30)
    kw = dict(red_src=fc.R_VECTOR, sem_src=fc.G_VECTOR, corr_src=fc.C_COSINE)
    fused, _ = P.run_v(cfg, None, ctx=ctx, **kw)
    staged, _ = P.run_v(cfg, None, ctx=ctx, staged=True, **kw)
    for k in fused:
        assert np.array_equal(fused[k], staged[k]), k


def test_v_step_long_rows_cosine_d_tail(ctx):
    """Feature width that is not a multiple of 8 (exact path) and one that is a multiple of 8
    but not of the matrix-core K step (zero-padded tail)."""
    for D in (52, 72, 200):
        cfg = synth.ficoco_v_single(seed=40 + D, B=2, grid=7, D=D, H=2, centres=4, dtype="bf16", n_keep=20)
        _check_v(cfg, ctx, corr_src=fc.C_COSINE)
