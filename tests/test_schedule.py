"""FLOPs model and reduction schedule (appendix "Theoretical FLOPs Calculation"; Sec.
"Implementation Details"): pins for the oracle's statement of the model, and the library's
host-side `ficoco_schedule` against it (no GPU involved: integer outputs must be equal)."""
import numpy as np
import pytest

from oracle import ficoco_oracle as O
from paper_2411_17686_amd import ficoco as fc


def test_layer_cost_closed_forms():
    # one token, D = F = 1: 4 + 2 + 2
    assert O.layer_flops(1, 1, 1) == 8.0
    # the three terms separately: linear in F, quadratic in the token count
    assert O.layer_flops(10, 8, 0) == 4 * 10 * 64 + 2 * 100 * 8
    assert O.layer_flops(10, 8, 5) - O.layer_flops(10, 8, 0) == 2 * 10 * 8 * 5
    n, s, D, F = 576, 64, 1024, 4096
    # before - after as the appendix defines the two: 4 s D^2 + 2 (2 n s - s^2) D + 2 s D F
    delta = O.layer_flops(n, D, F) - O.layer_flops(n - s, D, F)
    assert delta == 4.0 * s * D * D + 2.0 * (2 * n * s - s * s) * D + 2.0 * s * D * F
    # ... which is NOT the difference the appendix prints for the vision form (it lacks the
    # factor 2 on N N^S); recorded so that nobody "fixes" the model to match it
    printed = 4.0 * s * D * D + 2.0 * (n * s - s * s) * D + 2.0 * s * D * F
    assert delta - printed == 2.0 * n * s * D


def test_step_overhead_closed_forms():
    n, s, D = 576, 192, 1024
    v = O.step_flops("V", n, s, D)
    assert v == n * n + 2 * n + s * ((n - s) + 2 * D + 1) + D
    assert O.step_flops("L", n, s, D) - v == n * n + 2 * n          # the decoder form doubles the first bracket
    assert O.step_flops("V", n, 0, D) == n * n + 2 * n + D


def test_schedule_cost_by_hand():
    # 3 layers, reduction from layer 1 on, 10 tokens, 3 per layer, floor 5
    total, drops = O.schedule_cost("V", 3, 1, 10, 0, 4, 8, 5, 3)
    assert drops == [0, 3, 2]
    want = (O.layer_flops(10, 4, 8)
            + O.step_flops("V", 10, 3, 4) + O.layer_flops(7, 4, 8)
            + O.step_flops("V", 7, 2, 4) + O.layer_flops(5, 4, 8))
    assert total == want
    totalL, dropsL = O.schedule_cost("L", 3, 1, 10, 6, 4, 8, 5, 3)
    assert dropsL == drops
    assert totalL == (O.layer_flops(16, 4, 8) + O.step_flops("L", 10, 3, 4) + O.layer_flops(13, 4, 8)
                      + O.step_flops("L", 7, 2, 4) + O.layer_flops(11, 4, 8))


def test_schedule_is_the_smallest_count_within_budget():
    args = ("V", 24, 11, 576, 0, 1024, 4096, 16)
    full, _ = O.schedule_cost(*args, 0)
    ok, drops, total = O.schedule_uniform(*args, full)            # no reduction needed
    assert ok and drops == [0] * 24 and total == full
    ok, drops, total = O.schedule_uniform(*args, 0.8 * full)
    s = max(drops)
    assert ok and total <= 0.8 * full and s > 0
    prev, _ = O.schedule_cost(*args, s - 1)
    assert prev > 0.8 * full                                      # one token less per layer is too expensive
    assert drops[:11] == [0] * 11 and sum(drops) <= 576 - 16
    floor, _ = O.schedule_cost(*args, 576 - 16)
    ok, drops, total = O.schedule_uniform(*args, 0.5 * floor)     # unreachable: strongest schedule returned
    assert not ok and total == floor and drops[11] == 560


@pytest.mark.parametrize("seed", range(40))
def test_library_schedule_equals_oracle(seed):
    r = np.random.default_rng(900 + seed)
    variant = int(r.integers(0, 2))
    layers = int(r.integers(1, 40))
    start = int(r.integers(0, layers + 2))
    N = int(r.integers(1, 3000))
    M = int(r.integers(0, 600)) if variant else 0
    D = int(r.choice([1, 3, 64, 1024, 4096, 5120]))
    F = int(r.choice([1, 7, 256, 4096, 11008, 13824]))
    min_keep = int(r.integers(1, N + 1))
    v = "L" if variant else "V"
    full, _ = O.schedule_cost(v, layers, start, N, M, D, F, min_keep, 0)
    floor, _ = O.schedule_cost(v, layers, start, N, M, D, F, min_keep, N - min_keep)
    budget = float(r.choice([full, 0.999 * full, 0.7 * full + 0.3 * floor, 0.5 * (full + floor), floor,
                             0.9 * floor, 2.0 * full]))
    ok, drops, total = O.schedule_uniform(v, layers, start, N, M, D, F, min_keep, budget)
    rc, got, got_total = fc.ficoco_schedule(variant, layers, start, N, M, D, F, min_keep, budget)
    assert (rc == fc.OK) == ok
    assert got == drops
    assert got_total == total                    # same expressions in the same order: bit-equal doubles


def test_library_schedule_rejects_bad_arguments():
    for bad in (dict(layers=0), dict(N=0), dict(min_keep=0), dict(min_keep=11), dict(budget_flops=0.0),
                dict(variant=5), dict(D=0), dict(start_layer=-1)):
        kw = dict(variant=0, layers=4, start_layer=1, N=10, M=0, D=8, F=16, min_keep=2, budget_flops=1e9)
        kw.update(bad)
        with pytest.raises(fc.FicocoError):
            fc.ficoco_schedule(**kw)


def test_paper_scale_example():
    """CLIP ViT-L/14-336 encoder shape (24 layers, 576 patches, D = 1024, F = 4096), reduction
    from the 12th layer on: the schedule for 80 % of the unreduced cost."""
    full, _ = O.schedule_cost("V", 24, 11, 576, 0, 1024, 4096, 1, 0)
    rc, drops, total = fc.ficoco_schedule(fc.VARIANT_V, 24, 11, 576, 0, 1024, 4096, 1, 0.8 * full)
    assert rc == fc.OK and total <= 0.8 * full and len(set(drops[11:])) <= 2 and drops[:11] == [0] * 11
