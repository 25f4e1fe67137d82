"""Compile the HIP library ``libcpeval.so`` for gfx950, in-tree, with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcpeval.so")
SOURCES = ["graph.cpp", "cost.cpp", "api.hip", "kernels.hip", "window_shared.hip", "window_stream.hip", "column_slice.hip", "pct_order.hip", "constraints.hip", "search.hip", "simulate.hip"]
HEADERS = ["cpeval_internal.hpp", "launch.hpp", "device_math.hpp", os.path.join("..", "..", "include", "cpeval.h")]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return LIB
    cmd = [_hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Wall", "-Wno-unused-function",
           # packed-FP32 instruction forms are kept out of all device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True, cwd=CSRC)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
