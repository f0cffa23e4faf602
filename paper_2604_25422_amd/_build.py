"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libdwconv_gfx950.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # plain v_fma_f32 only
    "-ffp-contract=off",
    "-Wall", "-Wno-unused-command-line-argument",
    "-Wno-pass-failed",      # "#pragma unroll" on loops with run-time trip counts (long-filter kernels) is a hint only
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def dependencies():
    return sources() + sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(HERE, "..", "include", "dwconv.h")]


def build(verbose: bool = False, extra_flags=()) -> str:
    """Always recompiles; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-o", LIB_PATH] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in dependencies())


if __name__ == "__main__":
    print(build(verbose=True))
