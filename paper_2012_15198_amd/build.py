"""Builds the HIP library in-tree: paper_2012_15198_amd/libcxmix.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libcxmix.so")
CSRC = os.path.join(HERE, "csrc")
SOURCES = [os.path.join(CSRC, f) for f in ("cx_host.cpp", "cx_hbm.cpp", "cx_api_gossip.hip", "cx_api_hier.hip",
                                           "cx_api_pushsum.hip", "cx_api_fused.hip", "cx_api_hiersgd.hip",
                                           "cx_api_bf16.hip", "cx_api_f16.hip", "cx_api_hier16.hip",
                                           "cx_api_noalloc.hip", "cx_api_fused16.hip", "cx_api_pushsum16.hip")]
HEADERS = [os.path.join(ROOT, "include", "cx_mix.h")] + [os.path.join(CSRC, h) for h in (
    "cx_schedule.hpp", "cx_tile.hpp", "cx_ops.hpp", "cx_ops16.hpp", "cx_kernels.hpp", "cx_launch.hpp")]
OBJDIR = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
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
    os.makedirs(OBJDIR, exist_ok=True)
    objs = [os.path.join(OBJDIR, os.path.basename(src) + ".o") for src in SOURCES]

    def compile_one(pair):
        src, obj = pair
        cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), file=sys.stderr)
        subprocess.check_call(cmd)

    # one translation unit per entry point: compile them side by side, then link
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), int(os.environ.get("MAX_JOBS", "8")))) as pool:
        list(pool.map(compile_one, zip(SOURCES, objs)))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(link), file=sys.stderr)
    subprocess.check_call(link)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
