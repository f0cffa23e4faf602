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


# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch, FETCH_SIZE
# scaled by 2.00 and WRITE_SIZE by 1.00: what the same counters read for a plain 128 MiB device copy).
# Keyed by (workload index, kernel); the figures and the commands are in the text summaries under profiles/.
MEASURED_TRAFFIC_BYTES = {
    (1, "fwd"): 262325 * 1024, (1, "dx"): 262325 * 1024, (1, "dw_partial"): 268418 * 1024, (1, "bwd_fused"): 407515 * 1024,
    (2, "fwd"): 525294 * 1024, (2, "dx"): 525294 * 1024, (2, "dw_partial"): 539684 * 1024, (2, "bwd_fused"): 831299 * 1024,
    (3, "fwd"): 163881 * 1024, (3, "dx"): 163881 * 1024, (3, "dw_partial"): 271351 * 1024,
    (4, "fwd"): 393355 * 1024, (4, "dx"): 393355 * 1024, (4, "dw_partial"): 396139 * 1024, (4, "bwd_fused"): 598836 * 1024,
    (8, "fwd"): 69698 * 1024, (8, "dx"): 69698 * 1024, (8, "dw_partial"): 188048 * 1024,
    (7, "fwd"): 393537 * 1024, (7, "dx"): 393537 * 1024, (7, "dw_partial"): 394072 * 1024,
    (6, "fwd"): 262396 * 1024, (6, "dx"): 262396 * 1024, (6, "dw_partial"): 273273 * 1024,
    (5, "fwd"): 786611 * 1024, (5, "dx"): 786611 * 1024, (5, "dw_partial"): 786934 * 1024, (5, "bwd_fused"): 1234118 * 1024,
}


def measured_traffic(workload_index, kernel):
    """HBM bytes per launch from the committed rocprofv3 summaries, or None where none was taken."""
    return MEASURED_TRAFFIC_BYTES.get((workload_index, kernel))
