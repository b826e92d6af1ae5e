"""Seeded random sweep of small FiCoCo-V / FiCoCo-L problems over shapes, dtypes, score and
correlation sources, quantiles and ablation variants: every case is compared with the oracle to the
bars of tests/parity.py."""
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


@pytest.mark.parametrize("seed", range(60))
def test_random_v_case(ctx, seed):
    r = np.random.default_rng(5000 + seed)
    grid = int(r.integers(2, 15))
    N = grid * grid
    B = int(r.integers(1, 4))
    D = int(r.choice([1, 5, 8, 24, 33, 64, 130, 520]))
    H = int(r.integers(1, 6))
    n_keep = int(r.integers(1, N + 1))
    dtype = ["f32", "bf16"][seed % 2]
    mode = seed % 6
    cfg = synth.ficoco_v_single(seed=6000 + seed, B=B, grid=grid, D=D, H=H, centres=int(r.integers(1, 9)),
                                dtype=dtype, n_keep=n_keep)
    kw = {}
    if mode == 1:
        kw.update(corr_src=fc.C_COSINE)
    elif mode == 2:
        kw.update(red_src=fc.R_SIM_MEAN, sem_src=fc.G_EQ_TOKEN, corr_src=fc.C_COSINE)
    elif mode == 3:
        kw.update(k_mode=fc.K_FIXED, fixed_k=int(r.integers(0, 4)))
    elif mode == 4:
        kw.update(compress_mode=fc.COMPRESS_AVERAGE)
    elif mode == 5:
        kw.update(k_mode=fc.K_CONVERGENT)
    eps = float(r.choice([0.998, 1.0, 0.9, 0.5]))
    kw.update(eps=eps, k_max=64, window=int(r.choice([0, 2, 3])))
    out, _ = P.run_v(cfg, cfg["A"], ctx=ctx, **kw)
    okw = {k: v for k, v in kw.items() if k != "k_max"}
    extra = cfg["vis_begin"] + n_keep if (mode == 5 and n_keep < N) else None
    for b in range(B):
        ref = P.oracle_v(cfg, cfg["A"], b, **okw)
        if max([len(j) for j in ref["J"]] + [0]) > 64:       # more targets than the edge lists hold (ties, low quantiles)
            assert out["overflow"][b] == 1
            continue
        P.compare_image(out, b, ref, dtype, cfg["vis_begin"], kw.get("corr_src", fc.C_ATTN) == fc.C_ATTN, extra_row=extra)


@pytest.mark.parametrize("seed", range(20))
def test_random_l_case(ctx, seed):
    r = np.random.default_rng(7000 + seed)
    N = int(r.integers(2, 200))
    cfg = synth.ficoco_l_decoder(seed=8000 + seed, B=int(r.integers(1, 3)), n_sys=int(r.integers(0, 9)), N=N,
                                 M=int(r.choice([1, 3, 16, 70, 130])), D=int(r.choice([8, 40, 96, 264])),
                                 H=int(r.integers(1, 5)), centres=int(r.integers(1, 9)),
                                 n_keep=int(r.integers(1, N + 1)), with_vv=bool(seed % 2))
    red, cor = (fc.R_ATTN_RECV, fc.C_ATTN) if seed % 2 else (fc.R_SIM_MEAN, fc.C_COSINE)
    kw = [dict(), dict(k_mode=fc.K_FIXED, fixed_k=2), dict(compress_mode=fc.COMPRESS_AVERAGE)][seed % 3]
    out, _ = P.run_l(cfg, red, cor, ctx=ctx, **kw)
    for b in range(cfg["B"]):
        ref = P.oracle_l(cfg, b, red, cor, **kw)
        P.compare_image(out, b, ref, "bf16", cfg["vis_begin"], False)


def _run_v_case(ctx, cfg, dtype, kw, convergent=False):
    out, _ = P.run_v(cfg, cfg["A"], ctx=ctx, **kw)
    okw = {k: v for k, v in kw.items() if k != "k_max"}
    extra = cfg["vis_begin"] + cfg["n_keep"] if (convergent and cfg["n_keep"] < cfg["N"]) else None
    for b in range(cfg["B"]):
        ref = P.oracle_v(cfg, cfg["A"], b, **okw)
        if max([len(j) for j in ref["J"]] + [0]) > kw.get("k_max", 64):
            assert out["overflow"][b] == 1
            continue
        P.compare_image(out, b, ref, dtype, cfg["vis_begin"], kw.get("corr_src", fc.C_ATTN) == fc.C_ATTN, extra_row=extra)


@pytest.mark.parametrize("seed", range(15))
def test_random_medium_v_case(ctx, seed):
    """225 to 1444 patches, feature widths up to 1030 (several spans and a ragged tail): the shapes
    where the reduction's chunk grid, the map tile and the merge's spans have more than one piece."""
    r = np.random.default_rng(9000 + seed)
    grid = int(r.integers(15, 39))
    B, D, H = int(r.integers(1, 4)), int(r.choice([8, 64, 520, 1030])), int(r.integers(1, 5))
    n_keep = int(r.integers(1, grid * grid + 1))
    dtype = ["f32", "bf16"][seed % 2]
    cfg = synth.ficoco_v_single(seed=9500 + seed, B=B, grid=grid, D=D, H=H, centres=int(r.integers(1, 40)),
                                dtype=dtype, n_keep=n_keep)
    kw, mode = {}, seed % 5
    if mode == 1:
        kw.update(k_mode=fc.K_FIXED, fixed_k=int(r.integers(0, 4)))
    elif mode == 2:
        kw.update(compress_mode=fc.COMPRESS_AVERAGE)
    elif mode == 3:
        kw.update(k_mode=fc.K_CONVERGENT)
    elif mode == 4:
        kw.update(corr_src=fc.C_COSINE)
    kw.update(eps=float(r.choice([0.998, 1.0, 0.99])), k_max=64, window=int(r.choice([0, 2, 3])))
    _run_v_case(ctx, cfg, dtype, kw, convergent=mode == 3)


@pytest.mark.parametrize("seed", [3, 12, 27, 39])
def test_random_inverted_list_case(ctx, seed):
    """More than 1024 discarded tokens: the edge lists are inverted, long buckets get a workgroup."""
    r = np.random.default_rng(13000 + seed)
    grid = int(r.integers(36, 58))
    N = grid * grid
    D, H = int(r.choice([64, 520])), int(r.integers(1, 3))
    n_keep = int(r.integers(8, N - 1030))
    dtype = ["f32", "bf16"][seed % 2]
    cfg = synth.ficoco_v_single(seed=13500 + seed, B=1, grid=grid, D=D, H=H, centres=int(r.integers(1, 40)),
                                dtype=dtype, n_keep=n_keep, sigma=float(r.choice([0.5, 1.0, 3.0])))
    kw, mode = {}, seed % 4
    if mode == 1:
        kw.update(k_mode=fc.K_FIXED, fixed_k=int(r.integers(1, 4)))
    elif mode == 2:
        kw.update(compress_mode=fc.COMPRESS_AVERAGE)
    elif mode == 3:
        kw.update(corr_src=fc.C_COSINE)
    kw.update(eps=float(r.choice([0.998, 1.0, 0.99])), k_max=64, window=int(r.choice([0, 2])))
    _run_v_case(ctx, cfg, dtype, kw)


@pytest.mark.parametrize("seed,k_max", [(1, 4), (2, 5), (3, 7), (4, 8), (5, 13), (6, 12)])
def test_inverted_lists_with_short_rows(ctx, seed, k_max):
    """The inversion reads the edge lists slot by slot, four slots per load when the list length
    allows it: list lengths that are and are not multiples of four, rows partly filled."""
    r = np.random.default_rng(14000 + seed)
    grid = int(r.integers(36, 50))
    N = grid * grid
    n_keep = int(r.integers(8, min(N - 1030, 900)))
    dtype = ["f32", "bf16"][seed % 2]
    cfg = synth.ficoco_v_single(seed=14500 + seed, B=int(r.integers(1, 3)), grid=grid, D=int(r.choice([64, 136])),
                                H=int(r.integers(1, 3)), centres=int(r.integers(1, 40)), dtype=dtype, n_keep=n_keep)
    kw = dict(k_mode=fc.K_FIXED, fixed_k=int(r.integers(1, 4))) if seed % 3 == 0 else {}
    kw.update(eps=0.998, k_max=k_max, window=int(r.choice([0, 2])))
    _run_v_case(ctx, cfg, dtype, kw)
