#!/usr/bin/env python3
"""Benchmark of the fused FiCoCo-V step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload (BASELINE config 1, step 1 -- the shape the metric is quoted on): B = 16 images,
[CLS] + 24x24 patches (N = 576), D = 1024, 16 heads, bfloat16; keep 384 of 576.  One
"step" is one call of ficoco_v_step on the whole batch: attention reduction, score + local
penalty, top-K filter, correlate / threshold / weights, compress.  Inputs are synthetic,
seeded, resident in HBM before the timed region; the step rotates over several distinct
input sets whose total size exceeds the 256 MB on-die cache so that HBM is really read.

Prints ONE JSON line: tokens/s (B*N input visual tokens per step), plus
  roofline     : the attention-reduction kernel, algorithmic bytes per launch
                 (|A| read + single-precision head-mean map written) over its mean launch
                 time, measured here with HIP events on the launch stream (kernel alone,
                 back to back; the event-pair time of the same launch inside the pipelined
                 steps, which also spans waits for the other stream, is reported beside it);
  cpu_baseline : the CPU oracle timed on this host on a bounded sample of the same batch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
B, GRID, D, H, N_KEEP = 16, 24, 1024, 16, 384
N = GRID * GRID
N_SETS = 4


def make_sets(device, n_sets):
    """Config-1 recipe drawn on the GPU (bf16 clustered tokens, softmax of N(0,1.5^2) logits)."""
    import torch
    sets = []
    g = torch.Generator(device=device)
    g.manual_seed(1)
    for _ in range(n_sets):
        centres = torch.randn(B, 64, D, device=device, generator=g)
        pick = torch.randint(0, 64, (B, N), device=device, generator=g)
        X = torch.empty(B, N + 1, D, device=device)
        X[:, 0] = torch.randn(B, D, device=device, generator=g)
        X[:, 1:] = torch.gather(centres, 1, pick[..., None].expand(B, N, D)) \
            + 0.3 * torch.randn(B, N, D, device=device, generator=g)
        A = torch.empty(B, H, N + 1, N + 1, device=device, dtype=torch.bfloat16)
        for b in range(B):
            A[b] = torch.softmax(1.5 * torch.randn(H, N + 1, N + 1, device=device, generator=g), -1).to(torch.bfloat16)
        sets.append((X.to(torch.bfloat16).contiguous(), A))
    return sets


def traffic_from_profiles():
    """HBM bytes per launch of the reduction kernel from the committed counter summary."""
    path = os.path.join(ROOT, "profiles", "attn_reduce_c1_step1_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run five plain 1 GiB device-to-device copies (a kernel of known traffic "
                         "against which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled)")
    ap.add_argument("--streams", type=int, default=2,
                    help="HIP streams the independent steps are issued on, round-robin (each has its own "
                         "workspace and outputs); 1 = strictly one step after the other")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (the step shards over the batch with no "
                 "exchange; no multi-GPU figure is produced). Use --gpus 1.")

    import torch
    from paper_2411_17686_amd import ficoco as fc
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    ctx = fc.Context(0)
    sets = make_sets(dev, N_SETS)
    probs = [fc.make_problem(X, variant=fc.VARIANT_V, vis_begin=1, N=N, n_keep=N_KEEP, A=A, cls_index=0,
                             grid=(1, GRID, GRID), window=2, penalty_coef=2.0, w_score=0.35, eps=0.998,
                             k_max=8) for X, A in sets]
    buf = fc.Buffers(probs[0], dev, torch.bfloat16)
    n_str = max(1, args.streams)
    streams = [torch.cuda.Stream(device=dev) for _ in range(n_str)]        # default priority
    bufs = [buf] + [fc.Buffers(probs[0], dev, torch.bfloat16) for _ in range(n_str - 1)]

    def sync():
        torch.cuda.synchronize()

    def run_steps(k):
        # Successive steps are independent batches: step i goes to stream i mod n_str, so the
        # latency-bound tail of one step overlaps the bandwidth-bound head of the next.
        for i in range(k):
            with torch.cuda.stream(streams[i % n_str]):
                fc.ficoco_v_step(ctx, probs[i % N_SETS], bufs[i % n_str])

    run_steps(args.warmup)
    sync()
    t0 = time.perf_counter()
    run_steps(args.steps)
    sync()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = B * N / (dt / args.steps)
    assert all(int(b_.overflow.sum().item()) == 0 for b_ in bufs)

    # Dominant kernel inside the same pipelined region: the library records a HIP event pair
    # around every attention-reduction launch, on the stream the launch goes to.
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
             for _ in range(args.steps)]
    for i, (e0, e1) in enumerate(pairs):            # first record creates the underlying handle
        e0.record(streams[i % n_str])
        e1.record(streams[i % n_str])
    sync()
    for i in range(args.steps):
        e0, e1 = pairs[i]
        ctx.set_reduce_probe(e0.cuda_event, e1.cuda_event)
        with torch.cuda.stream(streams[i % n_str]):
            fc.ficoco_v_step(ctx, probs[i % N_SETS], bufs[i % n_str])
    ctx.set_reduce_probe(None, None)
    sync()
    reduce_ms = sum(e0.elapsed_time(e1) for e0, e1 in pairs) / args.steps
    k_launch = args.steps

    # The same kernel alone on one stream (nothing else on the GPU), for reference.
    stream = torch.cuda.current_stream(dev)
    for i in range(8):
        fc.ficoco_reduce(ctx, probs[i % N_SETS], buf)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    sync()
    e0.record(stream)
    for i in range(k_launch):
        fc.ficoco_reduce(ctx, probs[i % N_SETS], buf)
    e1.record(stream)
    sync()
    alone_ms = e0.elapsed_time(e1) / k_launch
    a_bytes = B * H * (N + 1) * (N + 1) * 2
    abar_bytes = B * N * N * 4
    algo_bytes = a_bytes + abar_bytes
    achieved = algo_bytes / (alone_ms * 1e-3) / 1e9
    step_bytes = algo_bytes + B * (N + 1) * D * 2 + B * (N_KEEP + 1) * D * 2 + B * (N - N_KEEP) * N_KEEP * 4

    out = {
        "metric": "FiCoCo-V tokens/sec (B=16,N=576,D=1024)", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "steps_per_s": 1e3 / ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "BASELINE config 1, step 1: FiCoCo-V fused step, B=16, [CLS]+576 patches, "
                               "D=1024, H=16, bf16 tokens and maps, keep 384 of 576, %d rotating input sets"
                               % N_SETS,
                   "decision_dtype": "f64", "streams": n_str},
        "step_algorithmic_bytes": step_bytes,
        "step_hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"kernel": "attn_reduce_kernel<bf16>", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic_from_profiles(), "algorithmic_bytes": algo_bytes,
                     "avg_launch_us": alone_ms * 1e3, "launches_timed": k_launch,
                     "timed_how": "HIP event pair around %d back-to-back launches of the kernel alone on "
                                  "the launch stream, inputs rotating" % k_launch,
                     "in_pipeline_event_us": reduce_ms * 1e3},
    }

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        sync()
        del src, dst

    if not args.no_cpu_baseline:
        from oracle import ficoco_oracle as O
        from paper_2411_17686_amd.synth import to_numpy
        X, A = sets[0]
        n_img = 2
        Xh = [O.widen(to_numpy(X[b])) for b in range(n_img)]
        Ah = [O.widen(to_numpy(A[b])) for b in range(n_img)]
        t0 = time.perf_counter()
        reps = 0
        while True:
            for b in range(n_img):
                O.v_step(Xh[b], Ah[b], cls_index=0, vis_begin=1, N=N, n_keep=N_KEEP, lam=0.35, eps=0.998,
                         grid=(1, GRID, GRID), window=2, coef=2.0)
            reps += 1
            el = time.perf_counter() - t0
            if el > 12.0:
                break
        out["cpu_baseline"] = {"value": reps * n_img * N / el, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                               "sample": "%d of the 16 images of input set 0, %d passes, float64 numpy oracle "
                                         "(single thread), %.1f s" % (n_img, reps, el)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
