"""Seeded synthetic inputs shaped like the paper's workloads.

These generators serve the tests, the smoke check and the benchmark.  They hold none of
the method's arithmetic: only random draws, a softmax to make row-stochastic attention
maps, and the cast to the storage type.  Everything is generated on the CPU with a seeded
torch generator (so the CPU checker and the GPU library read the same bits) and returned
as CPU tensors; the caller moves them to the device.

Workloads (stand-ins for the paper's models, Sec. "Implementation Details" / "Backbone
Details": CLIP ViT-L/14-336 grids of 24x24 patches plus [CLS], multi-crop high-resolution
grids, a 7B-class decoder's visual span with a short text instruction, multi-frame video):
token rows are Gaussian cluster centres plus per-token noise, which creates the redundancy
the method is meant to remove; attention maps are softmaxes of Gaussian logits.
"""
import math

import torch


def _gen(seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def _cast(t, dtype):
    return t.to(torch.bfloat16 if dtype == "bf16" else torch.float32).contiguous()


def to_numpy(t):
    """CPU/GPU tensor -> numpy array a CPU checker can widen: float32 as is, bfloat16 as its
    uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()


def clustered_tokens(g, B, n, D, centres, noise=0.3):
    """[B, n, D] fp32: each row = one of `centres` N(0, I) centres (chosen uniformly) plus
    N(0, noise^2) noise."""
    out = torch.empty(B, n, D, dtype=torch.float32)
    for b in range(B):
        c = torch.randn(centres, D, generator=g)
        pick = torch.randint(0, centres, (n,), generator=g)
        out[b] = c[pick] + noise * torch.randn(n, D, generator=g)
    return out


def ar1_field(g, crops, h, w, D, rho):
    """Unit-variance separable AR(1) field over each h x w crop, independent per feature:
    neighbouring cells share rho-correlated offsets.  Returns [crops*h*w, D]."""
    z = torch.randn(crops, h, w, D, generator=g)
    k = math.sqrt(1.0 - rho * rho)
    for c in range(1, w):
        z[:, :, c] = rho * z[:, :, c - 1] + k * z[:, :, c]
    for r in range(1, h):
        z[:, r] = rho * z[:, r - 1] + k * z[:, r]
    return z.reshape(crops * h * w, D)


def softmax_attention(g, B, H, nq, nk, sigma, dtype):
    """[B, H, nq, nk] row-softmax of N(0, sigma^2) logits, cast to `dtype`."""
    out = torch.empty(B, H, nq, nk, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)
    for b in range(B):
        logits = torch.randn(H, nq, nk, generator=g)
        if sigma != 1.0:
            logits *= sigma
        out[b] = torch.softmax(logits, dim=-1).to(out.dtype)
    return out


# ------------------------------------------------------------------------------ configs
def ficoco_v_single(seed=0, B=1, grid=24, D=1024, H=16, centres=48, dtype="f32",
                    sigma=1.0, n_keep=192):
    """Config 0: one FiCoCo-V step on [CLS] + grid x grid patches."""
    g = _gen(seed)
    N = grid * grid
    X = torch.empty(B, N + 1, D, dtype=torch.float32)
    X[:, 0] = torch.randn(B, D, generator=g)
    X[:, 1:] = clustered_tokens(g, B, N, D, centres)
    A = softmax_attention(g, B, H, N + 1, N + 1, sigma, dtype)
    return dict(X=_cast(X, dtype), A=A, B=B, H=H, D=D, n_tot=N + 1, vis_begin=1, N=N,
                cls_index=0, n_keep=n_keep, dtype=dtype, grid=(1, grid, grid), window=2,
                coef=2.0, lam=0.35, eps=0.998)


def ficoco_v_batched(seed=1, B=16, grid=24, D=1024, H=16, centres=64, dtype="bf16",
                     sigma=1.5, keeps=(384, 256, 192)):
    """Config 1: B images, successive reduction steps; a fresh attention map per step,
    sized for the tokens that survive the previous step.  `attention(step)` draws the
    map for one step lazily (the maps are large)."""
    g = _gen(seed)
    N = grid * grid
    X = torch.empty(B, N + 1, D, dtype=torch.float32)
    X[:, 0] = torch.randn(B, D, generator=g)
    X[:, 1:] = clustered_tokens(g, B, N, D, centres)
    sizes = [N] + list(keeps[:-1])

    def attention(step):
        gs = _gen(seed * 1000003 + 17 * (step + 1))
        n = sizes[step] + 1
        return softmax_attention(gs, B, H, n, n, sigma, dtype)

    return dict(X=_cast(X, dtype), attention=attention, B=B, H=H, D=D, vis_begin=1, N=N,
                cls_index=0, keeps=tuple(keeps), sizes=tuple(sizes), dtype=dtype,
                grid=(1, grid, grid), window=2, coef=2.0, lam=0.35, eps=0.998)


def ficoco_v_multicrop(seed=2, B=4, crops=5, grid=24, D=1024, H=16, centres=200,
                       dtype="bf16", rho=0.8, n_keep=640):
    """Config 2: high-resolution multi-crop grid; spatially correlated noise."""
    g = _gen(seed)
    N = crops * grid * grid
    X = torch.empty(B, N + 1, D, dtype=torch.float32)
    X[:, 0] = torch.randn(B, D, generator=g)
    for b in range(B):
        c = torch.randn(centres, D, generator=g)
        pick = torch.randint(0, centres, (N,), generator=g)
        X[b, 1:] = c[pick] + 0.3 * ar1_field(g, crops, grid, grid, D, rho)
    A = softmax_attention(g, B, H, N + 1, N + 1, 1.0, dtype)
    return dict(X=_cast(X, dtype), A=A, B=B, H=H, D=D, n_tot=N + 1, vis_begin=1, N=N,
                cls_index=0, n_keep=n_keep, dtype=dtype, grid=(crops, grid, grid), window=2,
                coef=2.0, lam=0.35, eps=0.998)


def ficoco_l_decoder(seed=3, B=8, n_sys=35, N=576, M=64, D=4096, H=32, centres=96,
                     dtype="bf16", n_keep=144, with_vv=False):
    """Config 3: decoder sequence = system + visual + text tokens.  A_tv = the visual
    columns of an unmasked softmax over the whole row for each text query.  with_vv adds
    the causal visual->visual block (row q sees keys 0 .. n_sys+q) from the same family."""
    g = _gen(seed)
    n_tot = n_sys + N + M
    X = torch.randn(B, n_tot, D, generator=g)
    X[:, n_sys:n_sys + N] = clustered_tokens(g, B, N, D, centres)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    A_tv = torch.empty(B, H, M, N, dtype=tdt)
    for b in range(B):
        p = torch.softmax(torch.randn(H, M, n_tot, generator=g), dim=-1)
        A_tv[b] = p[:, :, n_sys:n_sys + N].to(tdt)
    out = dict(X=_cast(X, dtype), A_tv=A_tv, A_vv=None, B=B, H=H, D=D, n_tot=n_tot,
               vis_begin=n_sys, N=N, text_begin=n_sys + N, M=M, n_keep=n_keep, dtype=dtype,
               beta=0.6, gamma=0.6, eps=0.998)
    if with_vv:
        A_vv = torch.empty(B, H, N, N, dtype=tdt)
        keys = torch.arange(n_sys + N)
        mask = keys[None, :] > (n_sys + torch.arange(N))[:, None]        # [N, n_sys+N]
        for b in range(B):
            logits = torch.randn(H, N, n_sys + N, generator=g)
            logits.masked_fill_(mask[None], float("-inf"))
            A_vv[b] = torch.softmax(logits, dim=-1)[:, :, n_sys:].to(tdt)
        out["A_vv"] = A_vv
    return out


def ficoco_v_video(seed=4, B=1, frames=16, grid=24, D=1024, H=16, centres=64, dtype="bf16",
                   step_noise=0.1, n_keep=1152):
    """Config 4: long visual context without a map: per-head received-attention and
    [CLS]-like vectors only; frame t = frame t-1 + N(0, step_noise^2)."""
    g = _gen(seed)
    n = grid * grid
    N = frames * n
    X = torch.empty(B, N, D, dtype=torch.float32)
    for b in range(B):
        f = clustered_tokens(g, 1, n, D, centres)[0]
        for t in range(frames):
            if t > 0:
                f = f + step_noise * torch.randn(n, D, generator=g)
            X[b, t * n:(t + 1) * n] = f
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    recv = torch.softmax(torch.randn(B, H, N, generator=g), dim=-1).to(tdt)
    sem = torch.softmax(torch.randn(B, H, N, generator=g), dim=-1).to(tdt)
    return dict(X=_cast(X, dtype), recv_vec=recv, sem_vec=sem, B=B, H=H, D=D, n_tot=N,
                vis_begin=0, N=N, cls_index=-1, n_keep=n_keep, dtype=dtype,
                grid=(frames, grid, grid), window=2, coef=2.0, lam=0.35, eps=0.998)
