"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfb_amd.so")
SOURCES = ["fb_kernels.hip", "fb_graph.cpp", "fb_sell.cpp", "fb_stream.cpp", "fb_pstream.cpp", "fb_api.cpp", "fb_leaky.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # never emit packed FP32 arithmetic
    "-Wall", "-Wno-unused-function", "-x", "hip",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "fb_internal.h"), os.path.join(HERE, "..", "include", "fb.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(verbose: bool = False) -> str:
    cmd = [HIPCC] + FLAGS + sources() + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
