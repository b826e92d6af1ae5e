#!/usr/bin/env python3
"""Benchmark of the fused FiCoCo step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1]

Default workload (BASELINE config 1, step 1 -- the shape the metric is quoted on): B = 16
images, [CLS] + 24x24 patches (N = 576), D = 1024, 16 heads, bfloat16; keep 384 of 576.  One
"step" is one call of ficoco_v_step / ficoco_l_step on the whole batch: attention reduction,
score + local penalty, top-K filter, correlate / threshold / weights, compress.  Inputs are
synthetic, seeded, resident in HBM before the timed region; steps rotate over several distinct
input sets whose total size exceeds the 256 MB on-die cache, and alternate between two HIP
streams (independent batches: the latency-bound tail of one step overlaps the bandwidth-bound
head of the next; --streams 1 runs them strictly one after the other).

Other workloads: --config 0, 2, 3 (decoder, no visual->visual map: mean-cosine + cosine
correlation), 3p (decoder with the causal visual->visual map: Algorithm 2 as printed), 4
(video, vectors + cosine correlation), 1c (config 1 tokens with the cosine correlation).

After the timed loop the last step of every stream is run again alone on one stream and its
outputs are compared bit for bit (`outputs_checked`); tests/test_gpu_pipeline.py checks the same
launch pattern on the same inputs against the CPU oracle.

Prints ONE JSON line: tokens/s (B*N input visual tokens per step), plus
  roofline     : the dominant kernel -- the attention-reduction kernel (HBM bound: |A| read +
                 single-precision head-mean map written, per launch) or, for the cosine
                 workloads, the bf16 MFMA tile kernel (2*B*N^S*N^T*D flops per launch) -- over
                 its mean launch time, measured here with HIP event pairs that the library
                 records around that launch on the launch stream, in a loop of that stage alone;
                 the event-pair time of the same launch inside the pipelined steps (which also
                 spans waits for the other stream) is reported beside it;
  cpu_baseline : the CPU oracle timed on this host on every sequence of input set 0, by one worker
                 process alone and by all workers at once (started before the GPU is initialised;
                 --no-cpu-baseline starts none: use it under rocprofv3).
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
MFMA_BF16_PEAK_TFLOPS = 2500.0


def _clustered(torch, g, dev, B, n, D, centres, noise=0.3):
    c = torch.randn(B, centres, D, device=dev, generator=g)
    pick = torch.randint(0, centres, (B, n), device=dev, generator=g)
    return torch.gather(c, 1, pick[..., None].expand(B, n, D)) + noise * torch.randn(B, n, D, device=dev, generator=g)


def _softmax_map(torch, g, dev, B, H, nq, nk, sigma, dt, mask=None, cols=None):
    out = torch.empty(B, H, nq, (cols[1] - cols[0]) if cols else nk, device=dev, dtype=dt)
    for b in range(B):
        logits = sigma * torch.randn(H, nq, nk, device=dev, generator=g)
        if mask is not None:
            logits.masked_fill_(mask, float("-inf"))
        p = torch.softmax(logits, -1)
        out[b] = (p[..., cols[0]:cols[1]] if cols else p).to(dt)
    return out


def make_workload(torch, fc, name, dev):
    """The BASELINE recipes drawn on the GPU (same distributions as the seeded CPU generators the
    parity tests use; several large input sets are needed quickly here)."""
    g = torch.Generator(device=dev)
    bf, f32 = torch.bfloat16, torch.float32
    W = dict(name=name)
    if name in ("1", "1c", "1q", "0", "2", "2q"):
        B, grid_g, H, D = {"1": (16, 1, 16, 1024), "1c": (16, 1, 16, 1024), "1q": (16, 1, 16, 1024), "0": (1, 1, 16, 1024),
                           "2": (4, 5, 16, 1024), "2q": (4, 5, 16, 1024)}[name]
        N = grid_g * 576
        keep = {"1": 384, "1c": 384, "1q": 384, "0": 192, "2": 640, "2q": 640}[name]
        dt = f32 if name == "0" else bf
        centres = {"1": 64, "1c": 64, "1q": 64, "0": 48, "2": 200, "2q": 200}[name]
        sigma = 1.5 if name in ("1", "1c", "1q") else 1.0
        n_sets = {"1": 4, "1c": 4, "1q": 4, "0": 16, "2": 1, "2q": 4}[name]
        g.manual_seed({"1": 1, "1c": 1, "1q": 1, "0": 0, "2": 2, "2q": 2}[name])
        d_head = 64
        sets = []
        for _ in range(n_sets):
            X = torch.empty(B, N + 1, D, device=dev)
            X[:, 0] = torch.randn(B, D, device=dev, generator=g)
            X[:, 1:] = _clustered(torch, g, dev, B, N, D, centres)
            if name in ("1q", "2q"):
                # queries and keys whose logits q.k / sqrt(d) are about N(0, sigma^2): the same family of maps
                Q = (torch.randn(B, H, N + 1, d_head, device=dev, generator=g) * sigma ** 0.5).to(bf)
                K = (torch.randn(B, H, N + 1, d_head, device=dev, generator=g) * sigma ** 0.5).to(bf)
                sets.append(dict(X=X.to(dt).contiguous(), Q=Q, K=K))
                continue
            A = _softmax_map(torch, g, dev, B, H, N + 1, N + 1, sigma, dt)
            sets.append(dict(X=X.to(dt).contiguous(), A=A))
        es = 2 if dt == bf else 4
        W.update(label="BASELINE config %s: FiCoCo-V fused step, B=%d, [CLS]+%d patches, D=%d, H=%d, %s, keep %d%s"
                 % (name[0] + (" step 1" if name[0] == "1" else ""), B, N, D, H, "bf16" if dt == bf else "f32", keep,
                    ", cosine correlation variant" if name == "1c" else
                    ", maps formed from queries and keys (d_head 64) inside the step" if name in ("1q", "2q") else ""),
                 B=B, N=N, D=D, H=H, keep=keep, dtype="bf16" if dt == bf else "f32", variant=fc.VARIANT_V, sets=sets,
                 kw=dict(vis_begin=1, N=N, n_keep=keep, cls_index=0, grid=(grid_g, 24, 24), window=2,
                         penalty_coef=2.0, w_score=0.35, eps=0.998, k_max=8,
                         corr_src=fc.C_COSINE if name == "1c" else fc.C_ATTN),
                 dominant="gram" if name == "1c" else "qk" if name in ("1q", "2q") else "reduce",
                 qk_elements=B * H * (N + 1) * (N + 1), d_head=d_head,
                 qk_bytes=2 * B * H * (N + 1) * d_head * 2 + B * N * N * 4,
                 reduce_bytes=B * H * (N + 1) * (N + 1) * es + (0 if name == "1c" else B * N * N * 4),
                 gram_flops=2.0 * B * (N - keep) * keep * D,
                 step_bytes=B * H * (N + 1) * (N + 1) * es + B * N * N * 4 + B * (N + 1) * D * es
                 + B * (keep + 1) * D * es + B * (N - keep) * keep * 4 if name not in ("1c", "1q", "2q") else None)
    elif name in ("3", "3p", "3b", "3bp", "3q", "3pq"):
        B, n_sys, N, M, D, H, keep = 8, 35, 576, 64, 4096, 32, 144
        from_qk = name in ("3q", "3pq")
        d_head = D // H
        if name in ("3b", "3bp"):                # the 13B decoder shape with a long instruction
            M, D, H = 512, 5120, 40
        n_tot = n_sys + N + M
        g.manual_seed(3)
        sets = []
        keys = torch.arange(n_sys + N, device=dev)
        mask = (keys[None, :] > (n_sys + torch.arange(N, device=dev))[:, None])[None]
        for _ in range(3):
            X = torch.randn(B, n_tot, D, device=dev, generator=g)
            X[:, n_sys:n_sys + N] = _clustered(torch, g, dev, B, N, D, 96)
            if from_qk:
                # the decoder layer's queries and keys (logits about N(0, 1)); the maps are causal
                Q = torch.randn(B, H, n_tot, d_head, device=dev, generator=g).to(bf)
                K = torch.randn(B, H, n_tot, d_head, device=dev, generator=g).to(bf)
                sets.append(dict(X=X.to(bf).contiguous(), Q=Q, K=K))
                continue
            A_tv = _softmax_map(torch, g, dev, B, H, M, n_tot, 1.0, bf, cols=(n_sys, n_sys + N))
            st = dict(X=X.to(bf).contiguous(), A_text=A_tv)
            if name in ("3p", "3bp"):
                st["A"] = _softmax_map(torch, g, dev, B, H, N, n_sys + N, 1.0, bf, mask=mask, cols=(n_sys, n_sys + N))
            sets.append(st)
        with_vv = name in ("3p", "3bp", "3pq")
        q_rows = N + M if with_vv else M
        W.update(label="%s%s: FiCoCo-L fused step, B=8, 35 system + 576 visual + %d text tokens, "
                       "D=%d, H=%d, bf16, keep 144%s"
                       % ("BASELINE config 3" if M == 64 else "13B decoder shape", "'" if with_vv else "", M, D, H,
                          (" (with the causal visual->visual map)" if with_vv
                           else " (no visual->visual map: mean-cosine + cosine correlation)")
                          + (", maps formed from the decoder layer's queries and keys (d_head %d) inside the step" % d_head
                             if from_qk else "")),
                 B=B, N=N, D=D, H=H, keep=keep, dtype="bf16", variant=fc.VARIANT_L, sets=sets,
                 kw=dict(vis_begin=n_sys, N=N, n_keep=keep, a_q_begin=n_sys, a_k_begin=n_sys, at_k_begin=n_sys,
                         w_score=0.6, gamma=0.6, eps=0.998, k_max=8, window=0, sem_src=fc.G_TEXT_ATTN,
                         **(dict(M=M) if from_qk else {}),
                         red_src=fc.R_ATTN_RECV if with_vv else fc.R_SIM_MEAN,
                         corr_src=fc.C_ATTN if with_vv else fc.C_COSINE),
                 dominant="qk" if from_qk else "reduce" if with_vv else "gram",
                 qk_elements=B * H * q_rows * n_tot, d_head=d_head, qk_long=True,
                 qk_bytes=2 * B * H * n_tot * d_head * 2 + B * N * M * 8 + (B * N * N * 4 if with_vv else 0),
                 reduce_bytes=B * H * N * N * 2 + B * N * N * 4 + B * H * M * N * 2,
                 gram_flops=2.0 * B * (N - keep) * keep * D, step_bytes=None)
    elif name == "4":
        B, frames, D, H, keep = 1, 16, 1024, 16, 1152
        N = frames * 576
        g.manual_seed(4)
        sets = []
        for _ in range(12):
            f = _clustered(torch, g, dev, 1, 576, D, 64)[0]
            X = torch.empty(B, N, D, device=dev)
            for t in range(frames):
                if t:
                    f = f + 0.1 * torch.randn(576, D, device=dev, generator=g)
                X[0, t * 576:(t + 1) * 576] = f
            rv = torch.softmax(torch.randn(B, H, N, device=dev, generator=g), -1).to(bf)
            sv = torch.softmax(torch.randn(B, H, N, device=dev, generator=g), -1).to(bf)
            sets.append(dict(X=X.to(bf).contiguous(), recv_vec=rv, sem_vec=sv))
        W.update(label="BASELINE config 4: FiCoCo-V fused step, B=1, 16 frames x 576 = 9216 tokens, D=1024, bf16, "
                       "per-head received / semantic vectors, cosine correlation on the matrix cores, keep 1152",
                 B=B, N=N, D=D, H=H, keep=keep, dtype="bf16", variant=fc.VARIANT_V, sets=sets,
                 kw=dict(vis_begin=0, N=N, n_keep=keep, cls_index=-1, grid=(frames, 24, 24), window=2,
                         penalty_coef=2.0, w_score=0.35, eps=0.998, k_max=8, red_src=fc.R_VECTOR,
                         sem_src=fc.G_VECTOR, corr_src=fc.C_COSINE),
                 dominant="gram", reduce_bytes=None, gram_flops=2.0 * B * (N - keep) * keep * D, step_bytes=None)
    else:
        sys.exit("bench.py: unknown --config %r" % name)
    return W


def issue_steps(torch, step_fn, ctx, probs, bufs, streams, k, start=0, before_step=None):
    """The launch pattern that is timed: step i of [start, start + k) goes to stream i mod
    len(streams) with that stream's buffers and reads input set i mod len(probs).  Successive
    steps are independent batches; one ctx serves all streams."""
    n_str, n_sets = len(streams), len(probs)
    for i in range(start, start + k):
        if before_step is not None:
            before_step(i)
        with torch.cuda.stream(streams[i % n_str]):
            step_fn(ctx, probs[i % n_sets], bufs[i % n_str])


OUTPUT_FIELDS = ("X_out", "pos_out", "keep_idx", "discard_idx", "edge_cnt", "edge_tgt", "edge_alpha", "scores", "overflow")


def last_steps_equal_eager(torch, fc, step_fn, ctx, probs, bufs, k, dev, tdt, start=0):
    """After issue_steps(..., k, start): the outputs each stream's buffers hold (its last step)
    against the same step run alone on the current stream into fresh buffers, bit for bit."""
    n_str, n_sets = len(bufs), len(probs)
    torch.cuda.synchronize()
    ok = True
    for si in range(n_str):
        mine = [i for i in range(start, start + k) if i % n_str == si]
        if not mine:
            continue
        last = mine[-1]
        ref = fc.Buffers(probs[last % n_sets], dev, tdt)
        step_fn(ctx, probs[last % n_sets], ref)
        torch.cuda.synchronize()
        # edge-list slots behind a row's count are never written: only the stored entries count
        live = torch.arange(ref.edge_tgt.shape[2], device=dev)[None, None, :] < ref.edge_cnt[:, :, None]
        for f in OUTPUT_FIELDS:
            got, want = getattr(bufs[si], f), getattr(ref, f)
            if f in ("edge_tgt", "edge_alpha"):
                got, want = torch.where(live, got, 0), torch.where(live, want, 0)
            ok = ok and bool(torch.equal(got, want))
    return ok


def traffic_from_profiles():
    """HBM bytes per launch of the reduction kernel (config 1) from the committed counter summary."""
    path = os.path.join(ROOT, "profiles", "attn_reduce_c1_step1_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def _oracle_worker(job):
    """Runs in a CPU worker process: the oracle step on this worker's sequences, round-robin, until
    `budget` seconds have passed (at least one pass over them).  Returns (sequences done, start, end)
    on the system-wide monotonic clock."""
    from oracle import ficoco_oracle as O
    seqs = [{k: (None if v is None else O.widen(v)) for k, v in sq.items()} for sq in job["seqs"]]
    kw, okw = job["kw"], job["okw"]
    done = 0
    t0 = time.monotonic()
    while True:
        for sq in seqs:
            if job["variant"] == "VQ":
                O.v_step_qk(sq["X"], sq["Q"], sq["K"], job["qk_scale"], cls_index=kw["cls_index"], vis_begin=kw["vis_begin"],
                            N=kw["N"], n_keep=kw["n_keep"], lam=kw["w_score"], eps=kw["eps"], grid=kw["grid"], window=2,
                            coef=2.0, **okw)
            elif job["variant"] == "V":
                O.v_step(sq["X"], sq["A"], cls_index=kw["cls_index"], vis_begin=kw["vis_begin"], N=kw["N"],
                         n_keep=kw["n_keep"], lam=kw["w_score"], eps=kw["eps"], grid=kw["grid"], window=2, coef=2.0,
                         recv_vec=sq["recv_vec"], sem_vec=sq["sem_vec"], red_src=job["red"], sem_src=job["sem"],
                         corr_src=job["cor"], **okw)
            else:
                O.l_step(sq["X"], sq["A"], sq["A_text"], vis_begin=kw["vis_begin"], N=kw["N"], n_keep=kw["n_keep"],
                         beta=kw["w_score"], gamma=kw["gamma"], eps=kw["eps"], red_src=job["red"], corr_src=job["cor"], **okw)
            done += 1
        if time.monotonic() - t0 > job["budget"]:
            break
    return done, t0, time.monotonic()


def start_cpu_pool():
    """Worker processes for the CPU baseline.  Must be called before anything initialises the GPU:
    a process that has may not start programs, and every worker is a freshly started interpreter."""
    import multiprocessing as mp
    from concurrent.futures import ProcessPoolExecutor
    n = max(1, min(16, os.cpu_count() or 1))       # the GPU machine's CPU share for one GPU is 16 cores
    os.environ.setdefault("OMP_NUM_THREADS", "1")
    # An executor never replaces a worker that died (it fails instead), and it has started all of
    # its workers once n tasks have been pending at the same time.
    pool = ProcessPoolExecutor(max_workers=n, mp_context=mp.get_context("spawn"))
    list(pool.map(time.sleep, [0.3] * n))
    return pool, n


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(W, pool, n_workers, budget=7.0):
    """The CPU oracle as it stands on every sequence of input set 0: one worker alone, then all
    workers at once (sequences dealt out round-robin)."""
    from paper_2411_17686_amd import ficoco as fc
    from paper_2411_17686_amd.synth import to_numpy
    st, kw = W["sets"][0], W["kw"]
    B = W["B"]

    def host(k, b):
        return None if st.get(k) is None else to_numpy(st[k][b])

    seqs = [dict(X=host("X", b), A=host("A", b), A_text=host("A_text", b), recv_vec=host("recv_vec", b),
                 sem_vec=host("sem_vec", b), Q=host("Q", b), K=host("K", b)) for b in range(B)]
    job = dict(variant=("VQ" if st.get("Q") is not None else "V") if W["variant"] == fc.VARIANT_V else "L",
               qk_scale=float(W.get("d_head", 64)) ** -0.5,
               kw={k: v for k, v in kw.items() if k in ("cls_index", "vis_begin", "N", "n_keep", "w_score", "eps", "grid", "gamma")},
               red={fc.R_ATTN_RECV: "attn", fc.R_VECTOR: "vector", fc.R_SIM_MEAN: "sim_mean"}[kw.get("red_src", fc.R_ATTN_RECV)],
               sem={fc.G_CLS_ATTN: "cls", fc.G_VECTOR: "vector", fc.G_TEXT_ATTN: "cls"}[kw.get("sem_src", fc.G_CLS_ATTN)],
               cor={fc.C_ATTN: "attn", fc.C_COSINE: "cosine"}[kw.get("corr_src", fc.C_ATTN)],
               okw=dict(k_mode={fc.K_ADAPTIVE: "adaptive", fc.K_FIXED: "fixed", fc.K_CONVERGENT: "convergent"}[kw.get("k_mode", 0)],
                        fixed_k=kw.get("fixed_k", 0), average=kw.get("compress_mode", 0) == fc.COMPRESS_AVERAGE),
               budget=budget)
    done1, t0, t1 = pool.submit(_oracle_worker, dict(job, seqs=seqs)).result()
    single = done1 * W["N"] / (t1 - t0)
    n_used = min(n_workers, B)
    shares = [dict(job, seqs=seqs[w::n_used]) for w in range(n_used)]
    res = list(pool.map(_oracle_worker, shares))
    wall = max(r[2] for r in res) - min(r[1] for r in res)
    done_all = sum(r[0] for r in res)
    return {"value": done_all * W["N"] / wall, "unit": "tokens/s", "cores": n_used, "kind": "oracle",
            "cpu_model": cpu_model(), "host_cores": os.cpu_count(),
            "sample": "all %d sequences of input set 0, dealt to %d worker processes (one numpy thread each) that "
                      "repeat the float64 numpy oracle on theirs for %.0f s: %d sequence-steps in %.1f s"
                      % (B, n_used, budget, done_all, wall),
            "single_thread": {"value": single, "unit": "tokens/s", "cores": 1,
                              "sample": "one worker, the %d sequences in turn for %.0f s: %d sequence-steps in %.1f s"
                                        % (B, budget, done1, t1 - t0)}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", default="1", help="0, 1 (default), 1c, 1q / 2q / 3q / 3pq (configs 1 / 2 / 3 / 3p with the maps formed from queries and keys), 2, 3, 3p, 4; "
                                                  "3b / 3bp: the 13B decoder shape")
    ap.add_argument("--ablation", default="none",
                    choices=["none", "fixed0", "fixed1", "fixed2", "convergent", "average"],
                    help="time one of the paper's ablation variants of the correlate / compress stages instead of "
                         "the method itself (not the headline figure)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run five plain 1 GiB device-to-device copies (a kernel of known traffic "
                         "against which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled)")
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams the independent steps are issued on, round-robin (each has its own "
                         "workspace and outputs); 1 = strictly one step after the other")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (the step shards over the batch with no "
                 "exchange; no multi-GPU figure is produced). Use --gpus 1.")

    # CPU workers for the oracle baseline are started first: nothing has touched the GPU yet.
    pool, n_workers = (None, 0) if args.no_cpu_baseline else start_cpu_pool()

    import torch
    from paper_2411_17686_amd import ficoco as fc
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    ctx = fc.Context(0)
    W = make_workload(torch, fc, args.config, dev)
    abl = {"none": {}, "fixed0": dict(k_mode=fc.K_FIXED, fixed_k=0), "fixed1": dict(k_mode=fc.K_FIXED, fixed_k=1),
           "fixed2": dict(k_mode=fc.K_FIXED, fixed_k=2), "convergent": dict(k_mode=fc.K_CONVERGENT),
           "average": dict(compress_mode=fc.COMPRESS_AVERAGE)}[args.ablation]
    W["kw"].update(abl)
    if abl:
        W["label"] += ", ablation variant %s" % args.ablation
    n_sets = len(W["sets"])
    probs = [fc.make_problem(st["X"], variant=W["variant"], A=st.get("A"), A_text=st.get("A_text"),
                             recv_vec=st.get("recv_vec"), sem_vec=st.get("sem_vec"), H=W["H"], Q=st.get("Q"), K=st.get("K"),
                             **W["kw"])
             for st in W["sets"]]
    tdt = torch.bfloat16 if W["dtype"] == "bf16" else torch.float32
    n_str = max(1, args.streams)
    streams = [torch.cuda.Stream(device=dev) for _ in range(n_str)]        # default priority
    bufs = [fc.Buffers(probs[0], dev, tdt) for _ in range(n_str)]
    step_fn = fc.ficoco_v_step if W["variant"] == fc.VARIANT_V else fc.ficoco_l_step
    sync = torch.cuda.synchronize
    # The inputs were drawn on the default stream and the side streams do not wait for it; the
    # buffers above may also sit in memory that temporaries of the generators (index tensors
    # among them) gave back to the allocator while kernels reading them are still queued.
    # Everything queued so far has to finish before a side stream touches any of it.
    sync()

    def run_steps(k, probe=None):
        hook = None
        if probe is not None:
            hook = lambda i: ctx.set_probe(probe[0], probe[1][i][0].cuda_event, probe[1][i][1].cuda_event)
        issue_steps(torch, step_fn, ctx, probs, bufs, streams, k, before_step=hook)
        if probe is not None:
            ctx.set_probe(probe[0], None, None)

    # Set-up, not warm-up: the first launch on a stream creates its hardware queue (milliseconds), so
    # every stream and input set is used once before the W warm-up steps and the timed region.
    run_steps(max(n_str, n_sets))
    sync()
    run_steps(args.warmup)
    sync()
    t0 = time.perf_counter()
    run_steps(args.steps)
    sync()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = W["B"] * W["N"] / (dt / args.steps)
    assert all(int(b_.overflow.sum().item()) == 0 for b_ in bufs)
    outputs_checked = last_steps_equal_eager(torch, fc, step_fn, ctx, probs, bufs, args.steps, dev, tdt)
    assert outputs_checked, "a pipelined step's outputs differ from the same step run alone"

    # Dominant kernel: event pairs recorded by the library around its launch.
    kind = fc.PROBE_REDUCE if W["dominant"] in ("reduce", "qk") else fc.PROBE_GRAM

    def event_pairs(n):
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for i, (e0, e1) in enumerate(pairs):            # the first record creates the underlying handle
            e0.record(streams[i % n_str])
            e1.record(streams[i % n_str])
        sync()
        return pairs

    pairs = event_pairs(args.steps)
    run_steps(args.steps, probe=(kind, pairs))          # (i) inside the pipelined steps
    sync()
    in_pipe_ms = sum(e0.elapsed_time(e1) for e0, e1 in pairs) / args.steps

    k_launch = args.steps                               # (ii) that stage alone on one stream
    pairs = event_pairs(k_launch)
    buf = bufs[0]
    with torch.cuda.stream(streams[0]):
        if kind == fc.PROBE_GRAM:                       # the correlate stage needs the earlier stages' state
            fc.ficoco_score(ctx, probs[0], buf)
            fc.ficoco_filter(ctx, probs[0], buf)
        for i in range(k_launch):
            ctx.set_probe(kind, pairs[i][0].cuda_event, pairs[i][1].cuda_event)
            if kind == fc.PROBE_REDUCE:
                fc.ficoco_reduce(ctx, probs[i % n_sets], buf)
            else:
                fc.ficoco_correlate(ctx, probs[0], buf)
        ctx.set_probe(kind, None, None)
    sync()
    alone = sorted(e0.elapsed_time(e1) for e0, e1 in pairs)
    # the same launches again, back to back, inside ONE event pair on the launch stream: the
    # average launch duration without the cost of recording an event around every launch
    span = event_pairs(1)[0]
    with torch.cuda.stream(streams[0]):
        span[0].record(streams[0])
        for i in range(k_launch):
            if kind == fc.PROBE_REDUCE:
                fc.ficoco_reduce(ctx, probs[i % n_sets], buf)
            else:
                fc.ficoco_correlate(ctx, probs[0], buf)
        span[1].record(streams[0])
    sync()
    alone_ms = span[0].elapsed_time(span[1]) / k_launch
    if kind == fc.PROBE_GRAM:
        # The correlate stage holds more than the Gram kernel, so one pair around whole calls will
        # not do; the library launches the kernel PROBE_REPEAT times in a row between its two
        # events instead (the launches write the same block), which spreads the cost of
        # recording the events over that many launches.
        k_rep = max(1, k_launch // 4)
        pairs_x = event_pairs(k_rep)
        with torch.cuda.stream(streams[0]):
            for i in range(k_rep):
                ctx.set_probe(fc.PROBE_GRAM_X16, pairs_x[i][0].cuda_event, pairs_x[i][1].cuda_event)
                fc.ficoco_correlate(ctx, probs[0], buf)
            ctx.set_probe(kind, None, None)
        sync()
        alone_ms = sum(e0.elapsed_time(e1) for e0, e1 in pairs_x) / (k_rep * fc.PROBE_REPEAT)
        k_launch = k_rep * fc.PROBE_REPEAT

    # (iii) latency of one fused step: event pairs around single calls, one stream, back to back
    lat_pairs = event_pairs(args.steps)
    with torch.cuda.stream(streams[0]):
        for i in range(args.steps):
            lat_pairs[i][0].record(streams[0])
            step_fn(ctx, probs[i % n_sets], bufs[0])
            lat_pairs[i][1].record(streams[0])
    sync()
    lat = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in lat_pairs)

    if W["dominant"] == "qk":
        # Arithmetic bound: per (image, head, query, key) seven single-precision vector operations
        # (scale, maximum, subtract, exponential, row sum, normalise, head accumulation) beside
        # 2 * d_head matrix-core flops; the vector operations are what the kernel waits for.
        algo = 7.0 * W["qk_elements"]
        achieved = algo / (alone_ms * 1e-3) / 1e12
        roof = {"kernel": "%s (softmax(QK^T) on bf16 MFMA 16x16x32, reduced on the fly)"
                          % ("attn_qk_long_kernel" if W.get("qk_long") or W["N"] + 1 > 640 else "attn_qk_kernel"), "bound": "alu",
                "achieved": achieved, "peak": 157.3, "unit": "TFLOP/s", "frac": achieved / 157.3, "traffic": None,
                "algorithmic_flops": algo, "mfma_flops": 2.0 * W["d_head"] * W["qk_elements"],
                "hbm_bytes_algorithmic": W["qk_bytes"],
                "note": "the materialised-map path reads %d bytes of maps for the same outputs (bench.py --config %s)"
                        % (W["qk_elements"] * 2, W["name"][0])}
    elif W["dominant"] == "reduce":
        algo = W["reduce_bytes"]
        achieved = algo / (alone_ms * 1e-3) / 1e9
        roof = {"kernel": "attn_reduce_kernel<%s>" % W["dtype"], "bound": "hbm", "achieved": achieved,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": traffic_from_profiles() if args.config == "1" else None,
                "traffic_source": "profiles/attn_reduce_c1_step1_pmc.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this "
                                  "kernel at this workload, scaled by a plain copy; read from that committed file, "
                                  "not measured in this run" if args.config == "1" else None,
                "algorithmic_bytes": algo}
    else:
        algo = W["gram_flops"]
        achieved = algo / (alone_ms * 1e-3) / 1e12
        gram_name = "gram_tile2_kernel" if args.config == "4" else "gram_tile_kernel"    # wide tiles from 128 blocks up
        roof = {"kernel": gram_name + " (bf16 MFMA 32x32x16)", "bound": "mfma", "achieved": achieved,
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                "traffic": None, "algorithmic_flops": algo}
    roof.update({"avg_launch_us": alone_ms * 1e3, "median_launch_us": alone[len(alone) // 2] * 1e3,
                 "launches_timed": k_launch,
                 "timed_how": ("one HIP event pair around %d back-to-back launches of the kernel alone on its stream "
                               "(median: event pairs recorded by the library around every launch)" % k_launch)
                 if kind == fc.PROBE_REDUCE else
                 ("HIP event pairs recorded by the library around runs of %d back-to-back launches of the kernel "
                  "(%d launches in all), that stage alone on one stream; median: pairs around single launches, "
                  "which include the cost of recording the events" % (fc.PROBE_REPEAT, k_launch)),
                 "in_pipeline_event_us": in_pipe_ms * 1e3})

    out = {
        "metric": ("FiCoCo-V tokens/sec (B=16,N=576,D=1024)" if args.config == "1"
                   else "FiCoCo tokens/sec (config %s)" % args.config)
                  + (", %d independent steps in flight on %d streams" % (n_str, n_str) if n_str > 1 else ", one step at a time"),
        "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "steps_per_s": 1e3 / ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": W["dtype"],
        "data": "synthetic",
        "config": {"workload": W["label"] + ", %d rotating input sets" % n_sets,
                   "decision_dtype": "f64", "streams": n_str},
        "roofline": roof,
    }
    out["outputs_checked"] = outputs_checked
    out["step_latency_us"] = {"median": lat[len(lat) // 2], "p10": lat[len(lat) // 10], "p90": lat[(9 * len(lat)) // 10],
                              "how": "HIP event pair around each of %d fused calls issued back to back on one stream" % len(lat)}
    one_us = lat[len(lat) // 2]
    out["one_stream"] = {"us_per_step": one_us, "steps_per_s": 1e6 / one_us, "tokens_per_s": W["B"] * W["N"] * 1e6 / one_us,
                         "how": "median of the fused calls issued back to back on one stream (no overlap between steps)"}
    if W.get("step_bytes"):
        # The whole fused step against the HBM roofline (the target is stated for the step, not for
        # its first kernel): algorithmic bytes of one step over the time of one step.
        out["step_algorithmic_bytes"] = W["step_bytes"]
        out["step_hbm_frac"] = W["step_bytes"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS
        out["step_roofline"] = {"bound": "hbm", "algorithmic_bytes": W["step_bytes"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                "frac_steps_in_flight": out["step_hbm_frac"],
                                "frac_one_step_at_a_time": W["step_bytes"] / (one_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                                "target_frac": 0.60}

    if args.config == "1" and args.ablation == "none":
        # BASELINE config 1 in full: the three successive reductions 576 -> 384 -> 256 -> 192 with a
        # fresh attention map per step (sized for the tokens the previous step left); X and the
        # position ids of a step are the previous step's outputs.  One chain per stream.
        keeps = (384, 256, 192)
        g = torch.Generator(device=dev)
        g.manual_seed(11)
        chains = []
        for si in range(n_str):
            ps, bs = [], []
            Xin, pos = W["sets"][si % n_sets]["X"], None
            n = W["N"]
            for k_i, keep in enumerate(keeps):
                A = W["sets"][si % n_sets]["A"] if k_i == 0 else _softmax_map(torch, g, dev, W["B"], W["H"], n + 1, n + 1, 1.5, tdt)
                kw = dict(W["kw"])
                kw.update(N=n, n_keep=keep)
                pr = fc.make_problem(Xin, variant=fc.VARIANT_V, A=A, H=W["H"], pos=pos, **kw)
                bf_ = fc.Buffers(pr, dev, tdt)
                ps.append((pr, A))
                bs.append(bf_)
                Xin, pos, n = bf_.X_out, bf_.pos_out, keep
            chains.append((ps, bs))
        sync()

        def run_chains(k):
            for i in range(k):
                ps, bs = chains[i % n_str]
                with torch.cuda.stream(streams[i % n_str]):
                    for (pr, _), bf_ in zip(ps, bs):
                        fc.ficoco_v_step(ctx, pr, bf_)

        k_chain = max(1, args.steps // 2)
        run_chains(max(1, args.warmup // 2))
        sync()
        t0 = time.perf_counter()
        run_chains(k_chain)
        sync()
        dtc = (time.perf_counter() - t0) / k_chain
        pair = event_pairs(k_chain)
        with torch.cuda.stream(streams[0]):
            for i in range(k_chain):
                pair[i][0].record(streams[0])
                for (pr, _), bf_ in zip(*chains[0]):
                    fc.ficoco_v_step(ctx, pr, bf_)
                pair[i][1].record(streams[0])
        sync()
        latc = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in pair)
        assert all(int(bf_.overflow.sum().item()) == 0 for _, bs in chains for bf_ in bs)
        out["three_step_chain"] = {"reductions": "576 -> 384 -> 256 -> 192 visual tokens, a fresh map per step",
                                   "us_per_chain": dtc * 1e6, "chains_per_s": 1.0 / dtc,
                                   "input_tokens_per_s": W["B"] * W["N"] / dtc,
                                   "one_chain_alone_us": latc[len(latc) // 2], "chains_timed": k_chain}

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        sync()
        del src, dst

    if pool is not None:
        out["cpu_baseline"] = cpu_baseline(W, pool, n_workers)
        pool.shutdown()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
