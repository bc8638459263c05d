"""Builds libsla.so (the C-ABI library) in-tree with hipcc for gfx950.

Usage:  python -m paper_2512_16093_amd.build
The library lands next to this file; tests, the smoke check and the benchmark
load it from there.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsla.so")
# The same library with the attention kernel's hand-counted copy waits replaced by full waits
# (-DSLA_FULL_WAITS): a checking build that a GPU test compares with the product build bit for bit.
LIB_FULL_WAITS = os.path.join(HERE, "libsla_fullwaits.so")
SOURCES = ["api.hip", "api_w8a8.hip", "k_classify.hip", "k_prep.hip", "k_linacc.hip", "k_sparse.hip", "k_w8a8.hip", "k_bwd.hip", "k_bwd_lin.hip", "k_calib.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         "-Wno-inline-asm"]  # (the asynchronous-copy helpers name m0 in their clobber lists on purpose)


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, err))
    if err.strip():
        sys.stderr.write(err + "\n")


def build(verbose=True):
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        _run([hipcc] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj])
        return src

    check_obj = os.path.join(objdir, "k_sparse_fullwaits.o")

    def check(_):
        _run([hipcc] + FLAGS + ["-DSLA_FULL_WAITS", "-c", os.path.join(CSRC, "k_sparse.hip"), "-o", check_obj])
        return "k_sparse.hip (-DSLA_FULL_WAITS)"

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        jobs = [ex.submit(one, pair) for pair in zip(SOURCES, objs)] + [ex.submit(check, None)]
        for j in jobs:
            name = j.result()
            if verbose:
                print("compiled", name, flush=True)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    k_sparse_obj = os.path.join(objdir, "k_sparse.o")
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_FULL_WAITS] +
         [check_obj if o == k_sparse_obj else o for o in objs])
    if verbose:
        print("linked", LIB, "and", LIB_FULL_WAITS, flush=True)
    return LIB


if __name__ == "__main__":
    build()
