"""The C-ABI library loads without a GPU, exports every function include/ficoco.h declares,
the ctypes mirror of `ficoco_problem` matches the C layout, and the host-side argument
checks behave (no kernel is launched here)."""
import ctypes as C
import os
import re
import subprocess
import sys

import pytest

from paper_2411_17686_amd import ficoco as fc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ficoco.h")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ficoco_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(fc.EXPORTS)
    L = fc.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert fc.lib().ficoco_version().decode().startswith("ficoco")


def test_problem_struct_layout_matches_header(tmp_path):
    """Compile the header with gcc and compare sizeof / offsetof with the ctypes mirror."""
    fields = [f[0] for f in fc.Problem._fields_]
    prog = ['#include <stdio.h>', '#include <stddef.h>', '#include "ficoco.h"', "int main(void){",
            'printf("%zu\\n", sizeof(ficoco_problem));']
    for f in fields:
        prog.append('printf("%%zu\\n", offsetof(ficoco_problem, %s));' % f)
    prog.append("return 0;}")
    src = tmp_path / "layout.c"
    src.write_text("\n".join(prog))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)])
    out = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    assert out[0] == C.sizeof(fc.Problem)
    for f, off in zip(fields, out[1:]):
        assert getattr(fc.Problem, f).offset == off, f


def _valid_problem():
    p = fc.Problem()
    p.variant, p.dtype = fc.VARIANT_V, fc.BF16
    p.B, p.H, p.D, p.n_tot, p.vis_begin, p.N, p.n_keep, p.cls_index = 16, 16, 1024, 577, 1, 576, 384, 0
    p.X, p.x_stride_b, p.x_stride_n = 4096, 577 * 1024, 1024
    p.A, p.a_stride_b, p.a_stride_h, p.a_stride_q = 8192, 16 * 577 * 577, 577 * 577, 577
    p.a_q_begin, p.a_nq, p.a_k_begin, p.a_nk = 0, 577, 0, 577
    p.grid_g, p.grid_h, p.grid_w, p.window, p.penalty_coef = 1, 24, 24, 2, 2.0
    p.w_score, p.gamma, p.eps = 0.35, 0.6, 0.998
    p.red_src, p.sem_src, p.corr_src, p.k_max = fc.R_ATTN_RECV, fc.G_CLS_ATTN, fc.C_ATTN, 8
    return p


def test_workspace_query_and_argument_checks():
    p = _valid_problem()
    n = fc.workspace_bytes(p)
    # at least the single-precision head-mean map and the inverted edge lists
    assert n >= 16 * 576 * 576 * 4 and n < 64 * 2 ** 20
    bad = [("n_keep", 577), ("n_keep", 0), ("eps", 1.5), ("k_max", 0), ("dtype", 7), ("N", 577),
           ("cls_index", 5), ("a_nk", 100), ("window", 2, "grid_h", 3), ("sem_src", fc.G_TEXT_ATTN),
           ("N", 20000), ("k_max", 20000)]
    for spec in bad:
        q = _valid_problem()
        for k, v in zip(spec[0::2], spec[1::2]):
            setattr(q, k, v)
        with pytest.raises(fc.FicocoError) as e:
            fc.workspace_bytes(q)
        assert e.value.code == fc.EINVAL, spec
    # FiCoCo-L needs the text block
    q = _valid_problem()
    q.variant, q.sem_src = fc.VARIANT_L, fc.G_TEXT_ATTN
    with pytest.raises(fc.FicocoError):
        fc.workspace_bytes(q)
    q.A_text, q.M, q.at_stride_b, q.at_stride_h, q.at_stride_q = 4096, 64, 1, 1, 576
    q.at_k_begin, q.at_nk = 1, 576
    assert fc.workspace_bytes(q) > n
    # Eq. 4's gamma is a convex weight: the candidate bounds of the correlate stage need 0 <= gamma <= 1
    for g in (-0.1, 1.5, float("nan")):
        q.gamma = g
        with pytest.raises(fc.FicocoError) as e:
            fc.workspace_bytes(q)
        assert e.value.code == fc.EINVAL
    q.gamma = 0.6
    # zero discards is legal
    q = _valid_problem()
    q.n_keep = 576
    assert fc.workspace_bytes(q) > 0


def test_product_path_has_no_oracle_import():
    """The binding and the kernels never reach into oracle/ (and the oracle never imports
    the package)."""
    pkg = os.path.join(ROOT, "paper_2411_17686_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            assert "paper_2411_17686_amd" not in open(os.path.join(ROOT, "oracle", f)).read()
