"""Builds libsccl.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libsccl.so")
SOURCES = [os.path.join(HERE, "csrc", "plan.cpp"), os.path.join(HERE, "csrc", "cost.cpp"),
           os.path.join(HERE, "csrc", "exec.hip")]
DEPS = SOURCES + [os.path.join(HERE, "csrc", "plan.hpp"), os.path.join(ROOT, "include", "sccl.h")]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source of the package into paper_2008_08708_amd/libsccl.so."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           "-ffp-contract=off", "-fno-fast-math",
           # packed fp32 instructions are kept out of every kernel of this library
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           "-x", "hip", *SOURCES, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def build_bench_kernels(verbose: bool = False) -> str:
    """Compile bench.py's measurement aids (plain streaming kernels of known traffic) into libbench_kernels.so
    beside bench.py.  They are not part of the library."""
    out = os.path.join(ROOT, "libbench_kernels.so")
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-x", "hip", os.path.join(ROOT, "bench_kernels.hip"), "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in DEPS)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_bench_kernels(verbose=True))
