"""Build libbload.so (the C-ABI HIP library) and libbload_yardsticks.so (plain streaming
kernels that a benchmark times beside it) in-tree for gfx950.

    python -m paper_2310_10879_amd.build

hipcc cross-compiles without a GPU present.  The shared objects land next to
this file so that the bindings, and a copy of the tree on another machine, find
them without any install step.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libbload.so")
YS_SRC = os.path.join(PKG, "yardsticks", "bload_yardsticks.hip")
YS_LIB = os.path.join(PKG, "libbload_yardsticks.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # keep the compiler from fusing float pairs into packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = True) -> str:
    cmd = [HIPCC] + FLAGS + ["-o", LIB] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    cmd = [HIPCC] + FLAGS + ["-o", YS_LIB, YS_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB, "and", YS_LIB)
    sys.exit(0)
