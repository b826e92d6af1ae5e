"""Builds the C-ABI library (and nothing else) in-tree with hipcc for gfx950.

    python -m paper_2411_17686_amd.build

The shared object lands next to this file as libficoco.so; the binding loads it from
there and raises if it is missing.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libficoco.so")
SOURCES = ["api.hip", "attn_reduce.hip", "attn_qk.hip", "select.hip", "correlate.hip", "compress.hip", "features.hip", "schedule.hip"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]


def build(verbose=True, out=LIB, defines=(), tag=""):
    """Compile every source and link `out`.  `defines` / `tag` build a tuning variant
    elsewhere without touching the product library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(HERE, "_build", src.replace(".hip", tag + ".o"))
        cmd = [hipcc, "-c"] + [f for f in FLAGS if f != "-shared"] + ["-D" + d for d in defines] \
            + ["-o", obj, os.path.join(CSRC, src)]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, pr in procs:
        log, _ = pr.communicate()
        log = "\n".join(l for l in log.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if pr.returncode != 0:
            failed = True
            sys.stderr.write("hipcc failed on %s:\n%s\n" % (src, log))
        elif verbose and log:
            sys.stderr.write(log + "\n")
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", out] + objs
    subprocess.check_call(cmd)
    if verbose:
        print("built", out)
    return out


def build_c_caller(verbose=True):
    """The plain-C caller of the ABI (tests/c_abi/step_check.c) as a shared object, with gcc."""
    root = os.path.dirname(HERE)
    src = os.path.join(root, "tests", "c_abi", "step_check.c")
    out = os.path.join(root, "tests", "c_abi", "libstep_check.so")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-Wall", "-shared", "-fPIC", "-I", os.path.join(root, "include"),
                           "-I", os.path.join(rocm, "include"), "-o", out, src, LIB, "-L" + os.path.join(rocm, "lib"),
                           "-lamdhip64", "-lm", "-Wl,-rpath," + HERE, "-Wl,-rpath," + os.path.join(rocm, "lib")])
    if verbose:
        print("built", out)
    return out


if __name__ == "__main__":
    build()
    build_c_caller()
