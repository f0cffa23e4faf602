"""Roofline bookkeeping (no operator arithmetic).

Operation counts follow the paper's roofline construction (Sec. III-G,
eqs. (flops_fwd_bwdin), (flops_bwdk), (roofline_metrics)); the byte counts are
the operator's own minimal traffic: every input read once, every output
written once.
"""
from __future__ import annotations


HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3    # dense fp32 matrix
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix
VALU_F32_PEAK_TFLOPS = 157.3    # 256 CU x 4 SIMD x 16 lanes x 2 (fma) x 2 (packed) x 2.4 GHz
VALU_F32_NONPACKED_TFLOPS = 78.6


def algorithmic_bytes(B, C, L, K, elem_size, path):
    """Bytes one path must move: two [B,C,L] tensors plus one [C,K] tensor."""
    n = B * C * L
    if path in ("fwd", "dx", "dw"):
        return (2 * n + C * K) * elem_size
    if path == "dw_partial":
        return 2 * n * elem_size
    if path == "step":
        return 3 * (2 * n + C * K) * elem_size
    raise ValueError(path)


def dense_flops(B, C, L, K):
    """Paper's count, eq. (flops_fwd_bwdin) = eq. (flops_bwdk): 2*K per output, padded taps included."""
    return 2 * B * C * L * K


def in_range_flops(B, C, L, K, pad_left):
    """2 flops per multiply-add whose input index falls inside [0, L)."""
    taps = 0
    for j in range(K):
        taps += max(0, L - abs(j - pad_left))
    return 2 * B * C * taps


# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE come from the text summaries under
# profiles/: every summary carries, per kernel, one line of the form
#     TRAFFIC workload=<index> kernel=<fwd|dx|dw_partial|bwd_fused> bytes=<n> sources=<a.h,b.h> digest=<12 hex digits>
# where digest is kernel_sources_digest(sources) at the time of the counter run.  A figure whose digest no longer
# matches the sources is stale and is not reported.
import glob
import hashlib
import os
import re

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_PROFILES = os.path.join(_HERE, "..", "profiles")
_TRAFFIC_RE = re.compile(r"TRAFFIC workload=(-?\d+) kernel=(\w+) bytes=(\d+) sources=([\w.,]+) digest=([0-9a-f]{12})")


def kernel_sources_digest(sources):
    """First 12 hex digits of the SHA-1 over the named files of csrc/ (sorted by name)."""
    h = hashlib.sha1()
    for name in sorted(sources):
        with open(os.path.join(_CSRC, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:12]


def measured_traffic(workload_index, kernel):
    """(bytes per launch, profile file name, stale?) from the committed rocprofv3 summaries; None where none was taken."""
    for path in sorted(glob.glob(os.path.join(_PROFILES, "*.md"))):
        with open(path) as f:
            text = f.read()
        for m in _TRAFFIC_RE.finditer(text):
            if int(m.group(1)) == workload_index and m.group(2) == kernel:
                try:
                    fresh = kernel_sources_digest(m.group(4).split(",")) == m.group(5)
                except OSError:
                    fresh = False
                return int(m.group(3)), os.path.basename(path), not fresh
    return None


if __name__ == "__main__":
    import sys
    print(kernel_sources_digest(sys.argv[1:]))
