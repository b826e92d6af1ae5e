"""The launch configuration bench.py times: three HIP streams, four rotating input sets, one ctx,
twelve fused steps in flight round-robin (bench.issue_steps, on bench.py's own inputs).  What every
stream's buffers hold at the end must equal (a) the same step run alone on one stream, bit for bit,
and (b) the CPU oracle, for one image of the input set that step read.  The other benchmark
configurations (cosine correlation with bucketed edges, FiCoCo-L, maps formed from queries and keys
with the head groups' partial sums in the workspace) are held to (a): every one of their kernels is
compared with the oracle on one stream elsewhere, what is new here is that three workspaces of one
context are in use at once."""
import pytest
import torch

from oracle import ficoco_oracle as O
from paper_2411_17686_amd import ficoco as fc
from paper_2411_17686_amd.synth import to_numpy
from tests import parity as P

pytestmark = pytest.mark.gpu


def test_pipelined_steps_on_three_streams_match_eager_and_oracle():
    import bench
    dev = torch.device("cuda", 0)
    ctx = fc.Context(0)
    W = bench.make_workload(torch, fc, "1", dev)        # BASELINE config 1 step 1, the benchmark's inputs
    probs = [fc.make_problem(st["X"], variant=W["variant"], A=st["A"], H=W["H"], **W["kw"]) for st in W["sets"]]
    assert len(probs) == 4
    streams = [torch.cuda.Stream(device=dev) for _ in range(3)]
    bufs = [fc.Buffers(probs[0], dev, torch.bfloat16) for _ in range(3)]
    torch.cuda.synchronize()                              # the inputs were drawn on the default stream
    kw = W["kw"]
    seen_sets = set()
    for start in (0, 1):
        bench.issue_steps(torch, fc.ficoco_v_step, ctx, probs, bufs, streams, 12, start=start)
        assert bench.last_steps_equal_eager(torch, fc, fc.ficoco_v_step, ctx, probs, bufs, 12, dev, torch.bfloat16, start=start)
        for si in range(3):
            last = [i for i in range(start, start + 12) if i % 3 == si][-1]
            st = W["sets"][last % 4]
            seen_sets.add(last % 4)
            b = (5 * si + 3 * start) % W["B"]
            ref = O.v_step(O.widen(to_numpy(st["X"][b])), O.widen(to_numpy(st["A"][b])), cls_index=kw["cls_index"],
                           vis_begin=kw["vis_begin"], N=kw["N"], n_keep=kw["n_keep"], lam=kw["w_score"], eps=kw["eps"],
                           grid=kw["grid"], window=kw["window"], coef=kw["penalty_coef"])
            P.compare_image(P.gpu_outputs(bufs[si]), b, ref, "bf16", kw["vis_begin"], True)
    assert seen_sets == {0, 1, 2, 3}
    ctx.close()


@pytest.mark.parametrize("config", ["4", "3", "1q", "3q"])
def test_pipelined_steps_of_the_other_configurations_match_eager(config):
    import bench
    dev = torch.device("cuda", 0)
    ctx = fc.Context(0)
    W = bench.make_workload(torch, fc, config, dev)
    probs = [fc.make_problem(st["X"], variant=W["variant"], A=st.get("A"), A_text=st.get("A_text"),
                             recv_vec=st.get("recv_vec"), sem_vec=st.get("sem_vec"), H=W["H"], Q=st.get("Q"),
                             K=st.get("K"), **W["kw"]) for st in W["sets"]]
    tdt = torch.bfloat16 if W["dtype"] == "bf16" else torch.float32
    step_fn = fc.ficoco_v_step if W["variant"] == fc.VARIANT_V else fc.ficoco_l_step
    streams = [torch.cuda.Stream(device=dev) for _ in range(3)]
    bufs = [fc.Buffers(probs[0], dev, tdt) for _ in range(3)]
    torch.cuda.synchronize()
    for start in (0, 1):
        bench.issue_steps(torch, step_fn, ctx, probs, bufs, streams, 12, start=start)
        assert bench.last_steps_equal_eager(torch, fc, step_fn, ctx, probs, bufs, 12, dev, tdt, start=start)
        assert all(int(b_.overflow.sum().item()) == 0 for b_ in bufs)
    ctx.close()
