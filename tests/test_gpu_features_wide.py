"""Long feature rows: 129, 257, 512, 640 and 1024 sixteen-byte vectors per row (the row kernels
read 64 vectors per step and wavefront, two to eight steps in flight, the last step partly
filled) and a token count that is no multiple of any row-chunk length -- with each
cosine-derived score term alone and both together, and with the cosine correlation (which reads
the bfloat16 unit rows) as well as the attention correlation."""
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


SOURCES = [(fc.R_SIM_MEAN, fc.G_EQ_TOKEN), (fc.R_SIM_MEAN, fc.G_CLS_ATTN), (fc.R_ATTN_RECV, fc.G_EQ_TOKEN),
           (fc.R_ATTN_RECV, fc.G_CLS_ATTN)]


@pytest.mark.parametrize("D", [1032, 2056, 4096, 5120, 8192])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_v_step_with_long_rows(ctx, D, dtype):
    for src, (red, sem) in enumerate(SOURCES):
        # the last pair scores from attention alone: with the cosine correlation the unit rows are then
        # formed by workgroups of the filter kernel's launch
        corr = fc.C_COSINE if src in (0, 3) else fc.C_ATTN
        cfg = synth.ficoco_v_single(seed=500 + D % 97 + src, B=2, grid=7, D=D, H=2, centres=5, dtype=dtype, n_keep=30)
        kw = dict(red_src=red, sem_src=sem, corr_src=corr, window=2, k_max=16)
        out, _ = P.run_v(cfg, cfg["A"], ctx=ctx, **kw)
        okw = {k: v for k, v in kw.items() if k != "k_max"}
        for b in range(cfg["B"]):
            ref = P.oracle_v(cfg, cfg["A"], b, **okw)
            P.compare_image(out, b, ref, dtype, cfg["vis_begin"], corr == fc.C_ATTN)


def test_decoder_step_scored_from_attention_with_cosine_correlation(ctx):
    """FiCoCo-L with the visual-to-visual map for the score and the cosine correlation for the merge
    (unit rows formed beside the filter), 70 text queries (statistics formed on the whole chip)."""
    cfg = synth.ficoco_l_decoder(seed=62, B=2, n_sys=2, N=77, M=70, D=2056, H=2, centres=6, n_keep=31, with_vv=True)
    for staged in (False, True):
        out, _ = P.run_l(cfg, fc.R_ATTN_RECV, fc.C_COSINE, ctx=ctx, staged=staged)
        for b in range(cfg["B"]):
            ref = P.oracle_l(cfg, b, fc.R_ATTN_RECV, fc.C_COSINE)
            P.compare_image(out, b, ref, cfg["dtype"], cfg["vis_begin"], False)


def test_decoder_step_with_long_rows(ctx):
    """FiCoCo-L without the visual-to-visual map (mean-cosine first term, cosine correlation) at the
    decoder's feature width, fused and staged."""
    cfg = synth.ficoco_l_decoder(seed=61, B=2, n_sys=3, N=83, M=9, D=4096, H=2, centres=6, n_keep=29, with_vv=False)
    for staged in (False, True):
        out, _ = P.run_l(cfg, fc.R_SIM_MEAN, fc.C_COSINE, ctx=ctx, staged=staged)
        for b in range(cfg["B"]):
            ref = P.oracle_l(cfg, b, fc.R_SIM_MEAN, fc.C_COSINE)
            P.compare_image(out, b, ref, cfg["dtype"], cfg["vis_begin"], False)
