"""Builds the HIP library in-tree: paper_2012_15198_amd/libcxmix.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libcxmix.so")
SOURCES = [os.path.join(HERE, "csrc", "cx_host.cpp"), os.path.join(HERE, "csrc", "cx_mix.hip")]
HEADERS = [os.path.join(ROOT, "include", "cx_mix.h")]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-ffp-contract=off",                      # the fp32 formulas are specified without FMA
    "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed fp32 math
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP/C++ source of the library for gfx950 (cross-compiles without a GPU)."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), *SOURCES, "-o", LIB]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
