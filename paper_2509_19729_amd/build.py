"""Builds libamoeba.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libamoeba.so")
SOURCES = ["api.cpp", "plan.cpp", "reshard_weights.hip", "reshard_kv.hip",
           "copy_baseline.hip", "merge_kv.hip"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the library cannot be built")
    return exe


def build(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  Always recompiles."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-Wno-unused-parameter",
           # keep the compiler from forming packed fp32 ops (no float math here, but the
           # flag is required for every HIP translation unit built for these boxes)
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-x", "hip"] + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
