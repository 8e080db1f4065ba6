"""Builds libsdl.so (HIP kernels + host plan, C ABI of include/sdl.h) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "csrc", f) for f in ("sdl_kernels.hip", "sdl_cosine.hip", "sdl_eval.hip", "sdl_plan.cpp", "sdl_engine.cpp",
                                                   "sdl_offload.cpp")]
LIB = os.path.join(HERE, "libsdl.so")

# -ffp-contract=off: every fp32 operation of the method rounds once, in the documented order.
# packed fp32 instructions are switched off for the test machines of machines.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-pass-failed", "-I", os.path.join(ROOT, "include")]


def build(verbose: bool = False, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *extra, "-o", LIB, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
