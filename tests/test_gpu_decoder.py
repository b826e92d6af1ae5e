"""GPU parity for the decoder-side use of a FiCoCo-L step: the selection applied to the key /
value cache and the position ids (Algorithm 2 removes the discarded tokens from the sequence the
following layers see), and the step at the 13B decoder shape (hidden size 5120, 40 heads, 512
text tokens)."""
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


def _problem_l(cfg, Xd, Atv, Avv, **kw):
    return fc.make_problem(
        Xd, variant=fc.VARIANT_L, vis_begin=cfg["vis_begin"], N=cfg["N"], n_keep=cfg["n_keep"],
        A=Avv, a_q_begin=cfg["vis_begin"], a_k_begin=cfg["vis_begin"], A_text=Atv, at_k_begin=cfg["vis_begin"],
        w_score=cfg["beta"], gamma=cfg["gamma"], eps=cfg["eps"],
        red_src=fc.R_ATTN_RECV if Avv is not None else fc.R_SIM_MEAN, sem_src=fc.G_TEXT_ATTN,
        corr_src=fc.C_ATTN if Avv is not None else fc.C_COSINE, k_max=8, window=0, **kw)


def test_gather_kv_cache_and_position_ids(ctx):
    cfg = synth.ficoco_l_decoder(seed=60, B=3, n_sys=7, N=120, M=20, D=96, H=4, centres=8, n_keep=33, with_vv=True)
    Xd, Atv, Avv = P.dev(cfg["X"]), P.dev(cfg["A_tv"]), P.dev(cfg["A_vv"])
    p = _problem_l(cfg, Xd, Atv, Avv)
    buf = fc.Buffers(p, "cuda", Xd.dtype)
    fc.ficoco_l_step(ctx, p, buf)
    n_tot = cfg["X"].shape[1]
    g = torch.Generator().manual_seed(5)
    kv = torch.randn(3, n_tot, 2, 4, 24, generator=g).to(torch.bfloat16)       # [B][n_tot][K|V][heads][dim]
    ids = torch.arange(n_tot, dtype=torch.int32).repeat(3, 1).contiguous()      # 4-byte rows: the narrow path
    odd = torch.randn(3, n_tot, 6, generator=g).to(torch.bfloat16)              # 12-byte rows
    strided = torch.randn(3, n_tot + 5, 40, generator=g)[:, 2:2 + n_tot, :32]   # row and batch strides
    outs = [fc.ficoco_gather_tokens(ctx, p, buf, t.to("cuda")) for t in (kv, ids, odd, strided)]
    torch.cuda.synchronize()
    keep = buf.keep_idx.cpu().numpy()
    for t, o in zip((kv, ids, odd, strided), outs):
        for b in range(3):
            want = O.gather_tokens(synth.to_numpy(t[b]) if t.dtype == torch.bfloat16 else t[b].numpy(),
                                   cfg["vis_begin"], cfg["N"], keep[b])
            got = synth.to_numpy(o[b].cpu()) if t.dtype == torch.bfloat16 else o[b].cpu().numpy()
            assert np.array_equal(got, want)
    # the token tensor itself, gathered, equals the step's pass-through rows where nothing was merged
    Xg = fc.ficoco_gather_tokens(ctx, p, buf, Xd)
    torch.cuda.synchronize()
    cnt = buf.edge_cnt.cpu().numpy(); tgt = buf.edge_tgt.cpu().numpy()
    for b in range(3):
        touched = {int(tgt[b, a, e]) for a in range(cnt.shape[1]) for e in range(cnt[b, a])}
        same = [r for r in range(Xg.shape[1]) if (r - cfg["vis_begin"]) not in touched]
        assert torch.equal(Xg[b, same], buf.X_out[b, same])


def test_gather_argument_errors(ctx):
    cfg = synth.ficoco_l_decoder(seed=61, B=1, n_sys=3, N=40, M=8, D=32, H=2, centres=4, n_keep=10, with_vv=True)
    Xd, Atv, Avv = P.dev(cfg["X"]), P.dev(cfg["A_tv"]), P.dev(cfg["A_vv"])
    p = _problem_l(cfg, Xd, Atv, Avv)
    buf = fc.Buffers(p, "cuda", Xd.dtype)
    fc.ficoco_l_step(ctx, p, buf)
    with pytest.raises(fc.FicocoError):                       # 2-byte rows
        fc.ficoco_gather_tokens(ctx, p, buf, torch.zeros(1, Xd.shape[1], 1, dtype=torch.bfloat16, device="cuda"))
    pc = _problem_l(cfg, Xd, Atv, Avv, k_mode=fc.K_CONVERGENT)
    with pytest.raises(fc.FicocoError) as e:
        fc.ficoco_gather_tokens(ctx, pc, buf, Xd, out=torch.empty_like(buf.X_out))
    assert e.value.code == fc.EUNSUPPORTED


@pytest.mark.parametrize("with_vv", [False, True])
def test_l_step_13b_decoder_shape(ctx, with_vv):
    """35 system + 576 visual + 512 text tokens, hidden size 5120, 40 heads (two sequences)."""
    cfg = synth.ficoco_l_decoder(seed=62, B=2, n_sys=35, N=576, M=512, D=5120, H=40, centres=96,
                                 n_keep=144, with_vv=with_vv)
    red, cor = (fc.R_ATTN_RECV, fc.C_ATTN) if with_vv else (fc.R_SIM_MEAN, fc.C_COSINE)
    out, _ = P.run_l(cfg, red, cor, ctx=ctx)
    assert out["X_out"].shape == (2, 35 + 144 + 512, 5120)
    for b in range(2):
        ref = P.oracle_l(cfg, b, red, cor)
        P.compare_image(out, b, ref, "bf16", cfg["vis_begin"], False)
