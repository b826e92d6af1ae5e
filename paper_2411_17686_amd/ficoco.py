"""Thin ctypes binding over libficoco.so (the C ABI declared in include/ficoco.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
torch is used for device memory (outputs, workspace) and for the current stream.  There is
no fallback: if the shared library has not been built, `lib()` raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libficoco.so")

OK, EINVAL, ENOMEM, EHIP, EUNSUPPORTED = 0, 1, 2, 3, 4
F32, BF16 = 0, 1
VARIANT_V, VARIANT_L = 0, 1
R_ATTN_RECV, R_VECTOR, R_SIM_MEAN = 0, 1, 2
G_CLS_ATTN, G_TEXT_ATTN, G_VECTOR, G_EQ_TOKEN = 0, 1, 2, 3
C_ATTN, C_COSINE = 0, 1
PROBE_REDUCE, PROBE_GRAM, PROBE_GRAM_X16 = 0, 1, 2
PROBE_REPEAT = 16
K_ADAPTIVE, K_FIXED, K_CONVERGENT = 0, 1, 2
COMPRESS_SELF, COMPRESS_AVERAGE = 0, 1

EXPORTS = ["ficoco_create", "ficoco_destroy", "ficoco_last_error", "ficoco_version",
           "ficoco_set_probe", "ficoco_workspace_bytes", "ficoco_out_rows", "ficoco_reduce", "ficoco_score",
           "ficoco_filter", "ficoco_correlate", "ficoco_correlation_gap", "ficoco_compress", "ficoco_v_step",
           "ficoco_l_step", "ficoco_schedule", "ficoco_gather_tokens", "ficoco_v_step_static"]
STATIC_SCRATCH_BYTES = 32 << 20


class Problem(C.Structure):
    """Mirror of `ficoco_problem` (field order and types must match the header)."""
    _fields_ = [
        ("variant", C.c_int32), ("dtype", C.c_int32),
        ("B", C.c_int32), ("H", C.c_int32), ("D", C.c_int32),
        ("n_tot", C.c_int32), ("vis_begin", C.c_int32), ("N", C.c_int32),
        ("n_keep", C.c_int32), ("cls_index", C.c_int32),
        ("X", C.c_void_p), ("x_stride_b", C.c_int64), ("x_stride_n", C.c_int64),
        ("A", C.c_void_p), ("a_stride_b", C.c_int64), ("a_stride_h", C.c_int64),
        ("a_stride_q", C.c_int64),
        ("a_q_begin", C.c_int32), ("a_nq", C.c_int32), ("a_k_begin", C.c_int32), ("a_nk", C.c_int32),
        ("A_text", C.c_void_p), ("at_stride_b", C.c_int64), ("at_stride_h", C.c_int64),
        ("at_stride_q", C.c_int64),
        ("M", C.c_int32), ("at_k_begin", C.c_int32), ("at_nk", C.c_int32),
        ("recv_vec", C.c_void_p), ("sem_vec", C.c_void_p),
        ("F", C.c_void_p), ("f_stride_b", C.c_int64), ("f_stride_n", C.c_int64), ("Df", C.c_int32),
        ("pos", C.c_void_p),
        ("grid_g", C.c_int32), ("grid_h", C.c_int32), ("grid_w", C.c_int32), ("window", C.c_int32),
        ("penalty_coef", C.c_float),
        ("w_score", C.c_float), ("gamma", C.c_float), ("eps", C.c_float),
        ("red_src", C.c_int32), ("sem_src", C.c_int32), ("corr_src", C.c_int32),
        ("k_max", C.c_int32),
        ("k_mode", C.c_int32), ("fixed_k", C.c_int32), ("compress_mode", C.c_int32),
        ("Q", C.c_void_p), ("K", C.c_void_p),
        ("qk_stride_b", C.c_int64), ("qk_stride_h", C.c_int64), ("qk_stride_n", C.c_int64),
        ("qk_begin", C.c_int32), ("qk_n", C.c_int32), ("d_head", C.c_int32), ("qk_dtype", C.c_int32),
        ("qk_scale", C.c_float),
    ]


class ScheduleProblem(C.Structure):
    """Mirror of `ficoco_schedule_problem`."""
    _fields_ = [("variant", C.c_int32), ("layers", C.c_int32), ("start_layer", C.c_int32),
                ("N", C.c_int32), ("M", C.c_int32), ("D", C.c_int32), ("F", C.c_int32),
                ("min_keep", C.c_int32), ("budget_flops", C.c_double)]


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libficoco.so is not built: run `python -m paper_2411_17686_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, i32p, f64p = C.c_void_p, C.c_void_p, C.c_void_p
        pp = C.POINTER(Problem)
        L.ficoco_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
        L.ficoco_destroy.argtypes = [C.c_void_p]
        L.ficoco_last_error.argtypes = [C.c_void_p]
        L.ficoco_last_error.restype = C.c_char_p
        L.ficoco_version.restype = C.c_char_p
        L.ficoco_set_probe.argtypes = [vp, C.c_int, vp, vp]
        L.ficoco_workspace_bytes.argtypes = [pp, C.POINTER(C.c_size_t)]
        L.ficoco_out_rows.argtypes = [pp, C.POINTER(C.c_int32)]
        L.ficoco_correlation_gap.argtypes = [vp, pp, vp, C.c_size_t, i32p, i32p, f64p, vp]
        L.ficoco_reduce.argtypes = [vp, pp, vp, C.c_size_t, vp]
        L.ficoco_score.argtypes = [vp, pp, vp, C.c_size_t, f64p, vp]
        L.ficoco_filter.argtypes = [vp, pp, vp, C.c_size_t, f64p, i32p, i32p, vp]
        L.ficoco_correlate.argtypes = [vp, pp, vp, C.c_size_t, i32p, i32p, i32p, i32p, f64p, i32p, vp]
        L.ficoco_compress.argtypes = [vp, pp, vp, C.c_size_t, i32p, i32p, i32p, i32p, f64p, vp, i32p, vp]
        step = [vp, pp, vp, C.c_size_t, vp, i32p, i32p, i32p, i32p, i32p, f64p, f64p, i32p, vp]
        L.ficoco_v_step.argtypes = step
        L.ficoco_l_step.argtypes = step
        L.ficoco_v_step_static.argtypes = step[:2] + step[4:]
        L.ficoco_gather_tokens.argtypes = [vp, pp, i32p, vp, C.c_int64, C.c_int64, C.c_int32, vp, vp]
        L.ficoco_schedule.argtypes = [C.POINTER(ScheduleProblem), C.POINTER(C.c_int32), C.POINTER(C.c_double)]
        for name in EXPORTS:
            getattr(L, name)            # fail loudly here if the build lacks a symbol
        _lib = L
    return _lib


class FicocoError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("ficoco status %d: %s" % (code, msg))
        self.code = code


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError("tokens and maps must be float32 or bfloat16")


class Context:
    """Owns a ficoco_ctx for one device."""

    def __init__(self, device=0):
        self._h = C.c_void_p()
        rc = lib().ficoco_create(C.byref(self._h), int(device))
        if rc != OK:
            raise FicocoError(rc, "ficoco_create failed")
        self.device = torch.device("cuda", int(device))

    def close(self):
        if self._h:
            lib().ficoco_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, rc):
        if rc != OK:
            raise FicocoError(rc, lib().ficoco_last_error(self._h).decode())

    def set_probe(self, kernel=PROBE_REDUCE, start_event=None, stop_event=None):
        """Raw hipEvent_t handles (ints) or None, None; see ficoco_set_probe."""
        self.check(lib().ficoco_set_probe(self._h, int(kernel), start_event, stop_event))

    def stream(self):
        return C.c_void_p(torch.cuda.current_stream(self.device).cuda_stream)


def make_problem(X, *, variant, vis_begin, N, n_keep, A=None, a_q_begin=0, a_k_begin=0,
                 cls_index=-1, A_text=None, at_k_begin=None, recv_vec=None, sem_vec=None, F=None,
                 pos=None, grid=(1, 0, 0), window=0, penalty_coef=2.0, w_score=0.35, gamma=0.6,
                 eps=0.998, red_src=R_ATTN_RECV, sem_src=G_CLS_ATTN, corr_src=C_ATTN, k_max=8, H=None,
                 k_mode=K_ADAPTIVE, fixed_k=0, compress_mode=COMPRESS_SELF, Q=None, K=None, qk_begin=0,
                 qk_scale=None, M=None):
    """Fill a `ficoco_problem` from torch tensors (shapes as in include/ficoco.h).  The
    returned Problem only holds raw pointers: keep the tensors alive while it is used."""
    p = Problem()
    p.variant = variant
    p.dtype = _dtype_code(X)
    B, n_tot, D = X.shape
    assert X.stride(2) == 1
    p.B, p.D, p.n_tot = B, D, n_tot
    p.vis_begin, p.N, p.n_keep, p.cls_index = vis_begin, N, n_keep, cls_index
    p.X, p.x_stride_b, p.x_stride_n = X.data_ptr(), X.stride(0), X.stride(1)
    heads = H
    if A is not None:
        assert A.dtype == X.dtype and A.stride(3) == 1
        heads = A.shape[1]
        p.A = A.data_ptr()
        p.a_stride_b, p.a_stride_h, p.a_stride_q = A.stride(0), A.stride(1), A.stride(2)
        p.a_q_begin, p.a_nq, p.a_k_begin, p.a_nk = a_q_begin, A.shape[2], a_k_begin, A.shape[3]
    if A_text is not None:
        assert A_text.dtype == X.dtype and A_text.stride(3) == 1
        heads = A_text.shape[1]
        p.A_text = A_text.data_ptr()
        p.at_stride_b, p.at_stride_h, p.at_stride_q = A_text.stride(0), A_text.stride(1), A_text.stride(2)
        p.M, p.at_nk = A_text.shape[2], A_text.shape[3]
        p.at_k_begin = vis_begin if at_k_begin is None else at_k_begin
    for name, v in (("recv_vec", recv_vec), ("sem_vec", sem_vec)):
        if v is not None:
            assert v.dtype == X.dtype and v.is_contiguous() and v.shape[0] == B and v.shape[2] == N
            heads = v.shape[1]
            setattr(p, name, v.data_ptr())
    p.H = int(heads) if heads is not None else 1
    if F is not None:
        assert F.dtype == X.dtype and F.stride(2) == 1
        p.F, p.f_stride_b, p.f_stride_n, p.Df = F.data_ptr(), F.stride(0), F.stride(1), F.shape[2]
    if pos is not None:
        assert pos.dtype == torch.int32 and pos.is_contiguous() and tuple(pos.shape) == (B, N)
        p.pos = pos.data_ptr()
    p.grid_g, p.grid_h, p.grid_w = grid
    p.window = window
    p.penalty_coef, p.w_score, p.gamma, p.eps = penalty_coef, w_score, gamma, eps
    p.red_src, p.sem_src, p.corr_src, p.k_max = red_src, sem_src, corr_src, k_max
    p.k_mode, p.fixed_k, p.compress_mode = k_mode, fixed_k, compress_mode
    if Q is not None:
        assert K is not None and Q.shape == K.shape and Q.stride() == K.stride() and Q.stride(3) == 1
        assert Q.dtype == torch.bfloat16 and K.dtype == torch.bfloat16 and Q.shape[0] == B
        p.Q, p.K = Q.data_ptr(), K.data_ptr()
        p.qk_stride_b, p.qk_stride_h, p.qk_stride_n = Q.stride(0), Q.stride(1), Q.stride(2)
        p.H = int(Q.shape[1])
        p.qk_begin, p.qk_n, p.d_head, p.qk_dtype = qk_begin, Q.shape[2], Q.shape[3], BF16
        p.qk_scale = float(Q.shape[3]) ** -0.5 if qk_scale is None else qk_scale
    if M is not None and A_text is None:
        p.M = M           # FiCoCo-L from queries and keys: the text tokens follow the visual span
    return p


def workspace_bytes(p):
    n = C.c_size_t()
    rc = lib().ficoco_workspace_bytes(C.byref(p), C.byref(n))
    if rc != OK:
        raise FicocoError(rc, "ficoco_workspace_bytes rejected the problem")
    return n.value


def out_rows(p):
    n = C.c_int32()
    rc = lib().ficoco_out_rows(C.byref(p), C.byref(n))
    if rc != OK:
        raise FicocoError(rc, "ficoco_out_rows rejected the problem")
    return n.value


class Buffers:
    """Output tensors and workspace for one problem shape (allocated once, reusable)."""

    def __init__(self, p, device, x_dtype):
        B, N, n_keep, k = p.B, p.N, p.n_keep, p.k_max
        n_disc = N - n_keep
        self.ws_bytes = workspace_bytes(p)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=device)
        off = (-self.ws.data_ptr()) % 256
        self.ws_ptr = self.ws.data_ptr() + off
        i32 = dict(dtype=torch.int32, device=device)
        self.X_out = torch.empty(B, out_rows(p), p.D, dtype=x_dtype, device=device)
        self.pos_out = torch.empty(B, n_keep, **i32)
        self.keep_idx = torch.empty(B, n_keep, **i32)
        self.discard_idx = torch.empty(B, max(n_disc, 1), **i32)[:, :n_disc]
        self.edge_cnt = torch.zeros(B, max(n_disc, 1), **i32)[:, :n_disc]
        self.edge_tgt = torch.zeros(B, max(n_disc, 1), k, **i32)[:, :n_disc]
        self.edge_alpha = torch.zeros(B, max(n_disc, 1), k, dtype=torch.float64, device=device)[:, :n_disc]
        self.scores = torch.empty(B, N, dtype=torch.float64, device=device)
        self.overflow = torch.zeros(B, **i32)
        self.gap = torch.zeros(B, max(n_disc, 1), dtype=torch.float64, device=device)[:, :n_disc]


def _ws(buf):
    return C.c_void_p(buf.ws_ptr), C.c_size_t(buf.ws_bytes)


def ficoco_reduce(ctx, p, buf):
    ws, n = _ws(buf)
    ctx.check(lib().ficoco_reduce(ctx._h, C.byref(p), ws, n, ctx.stream()))


def ficoco_score(ctx, p, buf):
    ws, n = _ws(buf)
    ctx.check(lib().ficoco_score(ctx._h, C.byref(p), ws, n, _ptr(buf.scores), ctx.stream()))


def ficoco_filter(ctx, p, buf):
    ws, n = _ws(buf)
    ctx.check(lib().ficoco_filter(ctx._h, C.byref(p), ws, n, _ptr(buf.scores), _ptr(buf.discard_idx),
                                  _ptr(buf.keep_idx), ctx.stream()))


def ficoco_correlate(ctx, p, buf):
    ws, n = _ws(buf)
    ctx.check(lib().ficoco_correlate(ctx._h, C.byref(p), ws, n, _ptr(buf.discard_idx), _ptr(buf.keep_idx),
                                     _ptr(buf.edge_cnt), _ptr(buf.edge_tgt), _ptr(buf.edge_alpha),
                                     _ptr(buf.overflow), ctx.stream()))


def ficoco_correlation_gap(ctx, p, buf):
    ws, n = _ws(buf)
    ctx.check(lib().ficoco_correlation_gap(ctx._h, C.byref(p), ws, n, _ptr(buf.discard_idx), _ptr(buf.keep_idx),
                                           _ptr(buf.gap), ctx.stream()))


def ficoco_compress(ctx, p, buf):
    ws, n = _ws(buf)
    ctx.check(lib().ficoco_compress(ctx._h, C.byref(p), ws, n, _ptr(buf.discard_idx), _ptr(buf.keep_idx),
                                    _ptr(buf.edge_cnt), _ptr(buf.edge_tgt), _ptr(buf.edge_alpha),
                                    _ptr(buf.X_out), _ptr(buf.pos_out), ctx.stream()))


def ficoco_gather_tokens(ctx, p, buf, t, out=None):
    """Rows of `t` [B][n_tot][...] (last axes contiguous) that survive the step in `buf`."""
    B, n_tot = t.shape[0], t.shape[1]
    row_bytes = t[0, 0].numel() * t.element_size()
    assert t[0, 0].is_contiguous() and B == p.B and n_tot == p.n_tot
    if out is None:
        out = torch.empty((B, out_rows(p)) + tuple(t.shape[2:]), dtype=t.dtype, device=t.device)
    ctx.check(lib().ficoco_gather_tokens(ctx._h, C.byref(p), _ptr(buf.keep_idx), _ptr(t),
                                         t.stride(0) * t.element_size(), t.stride(1) * t.element_size(),
                                         row_bytes, _ptr(out), ctx.stream()))
    return out


def _step(fn, ctx, p, buf):
    ws, n = _ws(buf)
    ctx.check(fn(ctx._h, C.byref(p), ws, n, _ptr(buf.X_out), _ptr(buf.pos_out), _ptr(buf.keep_idx),
                 _ptr(buf.discard_idx), _ptr(buf.edge_cnt), _ptr(buf.edge_tgt), _ptr(buf.edge_alpha),
                 _ptr(buf.scores), _ptr(buf.overflow), ctx.stream()))


def ficoco_v_step(ctx, p, buf):
    _step(lib().ficoco_v_step, ctx, p, buf)


def ficoco_l_step(ctx, p, buf):
    _step(lib().ficoco_l_step, ctx, p, buf)


def ficoco_v_step_static(ctx, p, buf):
    """ficoco_v_step on the library's static scratch: `buf.ws` is not used."""
    ctx.check(lib().ficoco_v_step_static(ctx._h, C.byref(p), _ptr(buf.X_out), _ptr(buf.pos_out), _ptr(buf.keep_idx),
                                         _ptr(buf.discard_idx), _ptr(buf.edge_cnt), _ptr(buf.edge_tgt),
                                         _ptr(buf.edge_alpha), _ptr(buf.scores), _ptr(buf.overflow), ctx.stream()))


def ficoco_schedule(variant, layers, start_layer, N, M, D, F, min_keep, budget_flops):
    """Per-layer discard counts within a FLOPs budget (host arithmetic; see ficoco_schedule).
    Returns (status, [n_discard per layer], total_flops); status is OK or EUNSUPPORTED."""
    sp = ScheduleProblem(variant, layers, start_layer, N, M, D, F, min_keep, budget_flops)
    out = (C.c_int32 * max(layers, 1))()
    total = C.c_double()
    rc = lib().ficoco_schedule(C.byref(sp), out, C.byref(total))
    if rc not in (OK, EUNSUPPORTED):
        raise FicocoError(rc, "ficoco_schedule rejected the arguments")
    return rc, list(out)[:layers], total.value
