"""The two cosine-derived score terms (mean cosine, equivalent token) on features that are
collinear without being identical: x_j = c * x_i.  In exact arithmetic such tokens tie; in
floating point they tie or differ in the last bits depending on the order of every sum.  The
library evaluates the terms fast and re-evaluates, in the defined order, the tokens whose
decision (window maximum, side of the top-K cut) lies within the error bound -- so the index
sets must equal the oracle's bit for bit here too."""
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


def _collinear_tokens(cfg, seed, scales):
    """Overwrite the visual rows: a few base rows (values with short mantissas, so that the
    multiples are exact in float32), every other row a multiple of one of them."""
    g = torch.Generator().manual_seed(seed)
    B, N, D = cfg["B"], cfg["N"], cfg["D"]
    X = cfg["X"].to(torch.float32).clone()
    n_base = max(2, N // 6)
    for b in range(B):
        base = torch.randn(n_base, D, generator=g).to(torch.bfloat16).to(torch.float32)
        base[base == 0] = 0.5
        pick = torch.randint(0, n_base, (N,), generator=g)
        c = torch.tensor(scales)[torch.randint(0, len(scales), (N,), generator=g)]
        rows = base[pick] * c[:, None]
        order = torch.randperm(N, generator=g)
        X[b, cfg["vis_begin"]:cfg["vis_begin"] + N] = rows[order]
    cfg["X"] = X.to(torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32).contiguous()
    return cfg


SOURCES = [(fc.R_SIM_MEAN, fc.G_EQ_TOKEN), (fc.R_SIM_MEAN, fc.G_CLS_ATTN), (fc.R_ATTN_RECV, fc.G_EQ_TOKEN)]


@pytest.mark.parametrize("D", [1, 8, 64])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("src", range(len(SOURCES)))
def test_scaled_duplicates_rank_as_in_the_oracle(ctx, D, dtype, src):
    red, sem = SOURCES[src]
    for window, scales in ((2, [1.0, 2.0, 0.5, 4.0]), (0, [1.0, 3.0, 1.5, 0.25, -2.0, 5.0])):
        cfg = synth.ficoco_v_single(seed=300 + 7 * D + src, B=2, grid=10, D=D, H=2, centres=4, dtype=dtype, n_keep=37)
        cfg = _collinear_tokens(cfg, 900 + D + src, scales)
        kw = dict(red_src=red, sem_src=sem, corr_src=fc.C_ATTN, window=window, k_max=16)
        out, _ = P.run_v(cfg, cfg["A"], ctx=ctx, **kw)
        okw = {k: v for k, v in kw.items() if k != "k_max"}
        for b in range(cfg["B"]):
            ref = P.oracle_v(cfg, cfg["A"], b, **okw)
            P.compare_image(out, b, ref, dtype, cfg["vis_begin"], True)


def test_identical_and_zero_rows(ctx):
    """All tokens identical (every score ties: the lowest indices are discarded) and a block of
    zero rows (cosine defined as 0)."""
    for variant in range(2):
        cfg = synth.ficoco_v_single(seed=77, B=1, grid=8, D=24, H=2, centres=3, dtype="bf16", n_keep=20)
        X = cfg["X"].clone()
        if variant == 0:
            X[:, 1:] = X[:, 1:2]
        else:
            X[:, 5:17] = 0
        cfg["X"] = X
        kw = dict(red_src=fc.R_SIM_MEAN, sem_src=fc.G_EQ_TOKEN, corr_src=fc.C_ATTN, window=2)
        out, _ = P.run_v(cfg, cfg["A"], ctx=ctx, **kw)
        ref = P.oracle_v(cfg, cfg["A"], 0, **kw)
        P.compare_image(out, 0, ref, "bf16", 1, True)
        if variant == 0:
            assert np.array_equal(ref["S"], np.arange(44)) or len(set(np.round(ref["scores"], 9))) > 1


def test_decoder_step_with_collinear_visual_tokens(ctx):
    """FiCoCo-L with the mean-cosine first term on collinear visual features (staged entry points:
    the score stage alone has to settle the ties the filter stage then sees)."""
    cfg = synth.ficoco_l_decoder(seed=55, B=2, n_sys=3, N=90, M=5, D=16, H=2, centres=4, n_keep=31, with_vv=True)
    cfg["dtype"] = "bf16"
    cfg = _collinear_tokens(cfg, 56, [1.0, 2.0, 0.5, 3.0])
    for staged in (False, True):
        out, _ = P.run_l(cfg, fc.R_SIM_MEAN, fc.C_ATTN, ctx=ctx, staged=staged)
        for b in range(cfg["B"]):
            ref = P.oracle_l(cfg, b, fc.R_SIM_MEAN, fc.C_ATTN)
            P.compare_image(out, b, ref, "bf16", cfg["vis_begin"], False)
