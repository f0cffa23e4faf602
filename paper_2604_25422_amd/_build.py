"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libdwconv_gfx950.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fvisibility=hidden",   # only the C ABI (DWCONV_API in include/dwconv.h) is exported
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # plain v_fma_f32 only
    "-ffp-contract=off",
    "-Wall", "-Wno-unused-command-line-argument",
    "-Wno-pass-failed",      # "#pragma unroll" on loops with run-time trip counts (long-filter kernels) is a hint only
]
OBJ_DIR = os.path.join(HERE, "_build")     # object files of the translation units (not tracked)


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def dependencies():
    return sources() + sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(HERE, "..", "include", "dwconv.h")]


def build(verbose: bool = False, extra_flags=(), jobs: int | None = None, incremental: bool = False) -> str:
    """Every translation unit to an object file (side by side), then one link.  Recompiles everything unless
    `incremental` (then only units older than their source or any header).  Returns the path of the shared library."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(OBJ_DIR, os.path.basename(p)[:-4] + ".o") for p in srcs]

    headers = sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(HERE, "..", "include", "dwconv.h")]
    newest_header = max(os.path.getmtime(h) for h in headers)

    def compile_one(pair):
        src, obj = pair
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            return
        cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    if jobs is None:
        jobs = max(1, min(len(srcs), os.cpu_count() or 1, 8))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(compile_one, zip(srcs, objs)))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in dependencies())


if __name__ == "__main__":
    import sys
    print(build(verbose=True, incremental="--incremental" in sys.argv))
