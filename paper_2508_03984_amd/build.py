"""Builds liboz2.so (the C-ABI library of include/oz2.h) for gfx950 with hipcc.

The library is built in-tree, next to this file, so that it travels with the
source tree; nothing is compiled at import time.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liboz2.so")
SOURCES = ["oz2_api.hip", "oz2_prepost.hip", "oz2_columns.hip", "oz2_small.hip", "oz2_accurate.hip", "oz2_int8_gemm.hip",
           "oz2_probe.hip", "oz2_constants.cpp"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # FMAs are written out where the method needs them
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build_library(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link liboz2.so; always rebuilds."""
    extra = os.environ.get("OZ2_EXTRA_HIPCC_FLAGS", "").split()      # for experiments
    cmd = [HIPCC] + FLAGS + extra + ["-x", "hip"] + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
