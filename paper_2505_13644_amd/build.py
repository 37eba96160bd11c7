"""Compile libctm.so (hand-written HIP for gfx950) in-tree with hipcc.

Usage:  python -m paper_2505_13644_amd.build        (or call build_library())
Objects go to _build/ at the repository root; the library lands next to this file.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libctm.so")
SOURCES = ["ctm_layer.hip", "ctm_layer_bf16.hip", "ctm_layer_bf16_t256.hip", "ctm_first.hip", "ctm_bwd.hip", "ctm_misc.hip", "ctm_small.hip", "ctm_api.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # loop heads on 32-byte boundaries: the stacked-GEMM k loop loses ~0.7 % when it straddles fetch windows
    "-falign-loops=32",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        raise RuntimeError("hipcc failed")
    return r.stderr


def build_library(verbose: bool = False, extra_flags=()) -> str:
    bdir = os.path.join(ROOT, "_build")
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]

    def one(i):
        return _run([HIPCC, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, SOURCES[i]), "-o", objs[i]])

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        logs = list(ex.map(one, range(len(SOURCES))))
    if verbose:
        sys.stderr.write("".join(logs))
    _run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB])
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
