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

# Kernels that prefetch into registers with loads the compiler does not track (inline assembly, one manual
# s_waitcnt before the registers are read): a spill or scratch copy of such a register between the load and the
# wait would read it before the data has arrived, so these kernels must not use scratch memory at all.
UNTRACKED_PREFETCH_KERNELS = ("corr_mfma_kernel", "corr_mfma_bf16_kernel", "corr_rowbatch_kernel", "dw_rowbatch_kernel",
                              "bwd_rowbatch_kernel", "corr_rowtall_kernel", "dw_rowtall_kernel")
VALIDATED_HIPCC = "7.2"       # ROCm release whose hipcc these kernels were checked with


def check_no_scratch(remarks: str, unit: str):
    """Parse -Rpass-analysis=kernel-resource-usage output; raise if a kernel with untracked prefetch uses scratch
    memory or accumulation registers (the compiler spills vector registers to either; a register it parks there
    between an untracked load and the manual wait would be saved before its data has arrived)."""
    import re
    name = None
    bad = []
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"(ScratchSize \[bytes/lane\]|AGPRs): (\d+)", line)
        if m and name and int(m.group(2)) > 0 and any(k in name for k in UNTRACKED_PREFETCH_KERNELS):
            bad.append((name, m.group(1), int(m.group(2))))
    if bad:
        raise RuntimeError(f"{unit}: kernels with untracked register prefetch must not spill, but use scratch memory or "
                           f"accumulation registers: {bad}")


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def dependencies():
    return sources() + sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(HERE, "..", "include", "dwconv.h")]


def build(verbose: bool = False, extra_flags=(), jobs: int | None = None, incremental: bool = False) -> str:
    """Every translation unit to an object file (side by side), then one link.  Recompiles everything unless
    `incremental` (then only units older than their source or any header).  Returns the path of the shared library."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    try:
        ver = subprocess.run([hipcc, "--version"], capture_output=True, text=True).stdout
        if f"HIP version: {VALIDATED_HIPCC}" not in ver:
            print(f"warning: kernels with untracked register prefetch were validated with hipcc {VALIDATED_HIPCC}; "
                  f"this is\n{ver.splitlines()[0] if ver else 'unknown'}", flush=True)
    except OSError:
        pass
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(OBJ_DIR, os.path.basename(p)[:-4] + ".o") for p in srcs]

    headers = sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(HERE, "..", "include", "dwconv.h")]
    newest_header = max(os.path.getmtime(h) for h in headers)

    def compile_one(pair):
        src, obj = pair
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            return
        cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        other = [ln for ln in r.stderr.splitlines() if "[-Rpass-analysis=kernel-resource-usage]" not in ln and
                 "is not a recognized feature for this target" not in ln]
        if other and (verbose or r.returncode != 0):
            print("\n".join(other), flush=True)
        if r.returncode != 0:
            raise subprocess.CalledProcessError(r.returncode, cmd)
        check_no_scratch(r.stderr, os.path.basename(src))

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
