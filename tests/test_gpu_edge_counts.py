"""More than 1024 discarded tokens, so the compress stage buckets the edges by target.  A fused step
counts the edges per target while the correlate stage writes the lists; a staged compress call counts
them from the lists it is handed.  Every kernel of the correlate stage that writes lists is driven
both ways here (sparse attention rows, candidate rows of FiCoCo-L, candidate rows behind the
matrix-core cosines, the general row kernel with lists longer than a wavefront and with materialised
rows), with several images per call."""
import pytest

from paper_2411_17686_amd import ficoco as fc
from paper_2411_17686_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = fc.Context(0)
    yield c
    c.close()


V_CASES = {
    "attention rows": dict(corr_src=fc.C_ATTN, k_max=8, eps=0.998),
    "cosine candidates": dict(corr_src=fc.C_COSINE, k_max=8, eps=0.998),
    "lists longer than a wavefront": dict(corr_src=fc.C_ATTN, k_max=80, eps=0.99),
    "materialised rows": dict(corr_src=fc.C_ATTN, k_max=64, eps=0.9),
    "materialised cosine rows": dict(corr_src=fc.C_COSINE, k_max=80, eps=0.95),
    "fixed two targets": dict(corr_src=fc.C_ATTN, k_max=8, eps=0.998, k_mode=fc.K_FIXED, fixed_k=2),
    "no targets": dict(corr_src=fc.C_ATTN, k_max=8, eps=0.998, k_mode=fc.K_FIXED, fixed_k=0),
}


@pytest.mark.parametrize("case", sorted(V_CASES))
@pytest.mark.parametrize("staged", [False, True])
def test_v_step_with_bucketed_edges(ctx, case, staged):
    kw = dict(V_CASES[case])
    dtype = "bf16" if len(case) % 2 else "f32"
    # 41 x 41 patches, 1681 - 470 = 1211 discarded rows: three shares of rows, the last one shorter
    cfg = synth.ficoco_v_single(seed=700 + len(case), B=3, grid=41, D=72, H=2, centres=7, dtype=dtype, n_keep=470)
    out, _ = P.run_v(cfg, cfg["A"], ctx=ctx, window=2, staged=staged, **kw)
    okw = {k: v for k, v in kw.items() if k != "k_max"}
    for b in range(cfg["B"]):
        ref = P.oracle_v(cfg, cfg["A"], b, window=2, **okw)
        assert max([len(j) for j in ref["J"]] + [0]) <= kw["k_max"]
        P.compare_image(out, b, ref, dtype, cfg["vis_begin"], kw["corr_src"] == fc.C_ATTN)


@pytest.mark.parametrize("corr", [fc.C_ATTN, fc.C_COSINE])
@pytest.mark.parametrize("M", [9, 40])
@pytest.mark.parametrize("staged", [False, True])
def test_decoder_step_with_bucketed_edges(ctx, corr, M, staged):
    cfg = synth.ficoco_l_decoder(seed=71 + M, B=2, n_sys=3, N=1500, M=M, D=64, H=2, centres=9, n_keep=260,
                                 with_vv=True)
    out, _ = P.run_l(cfg, fc.R_ATTN_RECV, corr, ctx=ctx, staged=staged)
    for b in range(cfg["B"]):
        ref = P.oracle_l(cfg, b, fc.R_ATTN_RECV, corr)
        P.compare_image(out, b, ref, cfg["dtype"], cfg["vis_begin"], corr == fc.C_ATTN)


@pytest.mark.parametrize("D", [64, 1544])
def test_more_long_buckets_than_workgroups_for_them(ctx, D):
    """2204 discarded tokens with three targets each among 100 preserved ones: nearly every target has
    more than 32 sources, and the merge has one workgroup per four possible such targets (at least 64),
    so some workgroups take a second target; 1544 features are two spans of a row."""
    cfg = synth.ficoco_v_single(seed=93, B=2, grid=48, D=D, H=2, centres=5, dtype="bf16", n_keep=100)
    kw = dict(corr_src=fc.C_ATTN, k_max=4, k_mode=fc.K_FIXED, fixed_k=3, window=2)
    out, _ = P.run_v(cfg, cfg["A"], ctx=ctx, **kw)
    okw = {k: v for k, v in kw.items() if k != "k_max"}
    for b in range(cfg["B"]):
        ref = P.oracle_v(cfg, cfg["A"], b, **okw)
        sizes = {}
        for j in ref["J"]:
            for t in j:
                sizes[int(t)] = sizes.get(int(t), 0) + 1
        assert sum(1 for v in sizes.values() if v > 32) > 64
        P.compare_image(out, b, ref, "bf16", cfg["vis_begin"], True)
