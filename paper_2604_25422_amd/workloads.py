"""Seeded synthetic inputs for the depthwise-convolution hot path.

This module holds no arithmetic of the operator itself: it only draws the
tensors that both the HIP library and the CPU checker are fed.  The shapes are
the five benchmark configurations of this build (index 1 is the headline
training-step shape) plus, as index 5, the shape of the paper's own measurements
(Sec. V: B = 16384, H = 128, L = 48, K = 48, pad K/2); seeded random tensors stand in for the S4ConvD
activations of the paper's ASHRAE GEPIII workload (Sec. III-A..C), whose
kernel time depends on tensor dimensions only (Sec. III-H).

All draws come from ``torch.Generator(device="cpu")``: seed ``BASE_SEED + i``
for x, ``+100`` for w, ``+200`` for dY, where ``i`` is the configuration index.
"""
from __future__ import annotations

import dataclasses
import math

import torch

BASE_SEED = 20260425


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int            # position in the configuration list (seeds derive from it)
    B: int
    C: int
    L: int
    K: int
    pad_left: int
    dtype: str            # "f32" | "bf16"  (storage type)
    w_kind: str           # "normal" | "normal_var_1_over_K" | "decay_cos"

    @property
    def N(self) -> int:
        return self.B * self.C * self.L

    @property
    def elem_size(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def with_shape(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


WORKLOADS = [
    Workload("cfg0_small_B4_C64_L1024_K16_causal_f32", 0, 4, 64, 1024, 16, 15, "f32", "normal"),
    Workload("cfg1_headline_B32_C256_L4096_K64_causal_f32", 1, 32, 256, 4096, 64, 63, "f32", "normal_var_1_over_K"),
    Workload("cfg2_shortK_B64_C512_L2048_K7_same_f32", 2, 64, 512, 2048, 7, 3, "f32", "normal"),
    Workload("cfg3_longK_B8_C256_L8192_K8192_causal_f32", 3, 8, 256, 8192, 8192, 8191, "f32", "decay_cos"),
    Workload("cfg4_bf16_B128_C768_L1024_K32_causal_bf16", 4, 128, 768, 1024, 32, 31, "bf16", "normal"),
    Workload("paper_shape_B16384_C128_L48_K48_pad24_f32", 5, 16384, 128, 48, 48, 24, "f32", "normal_var_1_over_K"),
    # not a configuration of the baseline file: a filter between the two classes it names (nine block offsets)
    Workload("midK_B32_C256_L4096_K128_causal_f32", 6, 32, 256, 4096, 128, 127, "f32", "normal_var_1_over_K"),
    # ... and the same filter length on bf16 storage at the bf16 geometry
    Workload("midK_B128_C768_L1024_K128_causal_bf16", 7, 128, 768, 1024, 128, 127, "bf16", "normal_var_1_over_K"),
    # ... and the long-filter configuration on bf16 storage
    Workload("longK_B8_C256_L8192_K8192_causal_bf16", 8, 8, 256, 8192, 8192, 8191, "bf16", "decay_cos"),
]
HEADLINE = WORKLOADS[1]


def torch_dtype(wl: Workload):
    return torch.float32 if wl.dtype == "f32" else torch.bfloat16


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def make_filter(wl: Workload) -> torch.Tensor:
    """w [C, K] in the workload's storage dtype."""
    g = _gen(BASE_SEED + wl.index + 100)
    if wl.w_kind == "normal":
        w = torch.randn(wl.C, wl.K, generator=g, dtype=torch.float32)
    elif wl.w_kind == "normal_var_1_over_K":
        w = torch.randn(wl.C, wl.K, generator=g, dtype=torch.float32) / math.sqrt(wl.K)
    elif wl.w_kind == "decay_cos":
        # w[c,k] = exp(-a_c k) cos(b_c k), k the array index; a ~ U(1e-4, 1e-2), b ~ U(0, pi);
        # evaluated in fp64, then rounded to fp32.
        a = 1e-4 + (1e-2 - 1e-4) * torch.rand(wl.C, generator=g, dtype=torch.float64)
        b = math.pi * torch.rand(wl.C, generator=g, dtype=torch.float64)
        k = torch.arange(wl.K, dtype=torch.float64)
        w = (torch.exp(-a[:, None] * k[None, :]) * torch.cos(b[:, None] * k[None, :])).to(torch.float32)
    else:
        raise ValueError(wl.w_kind)
    return w.to(torch_dtype(wl)).contiguous()


def make_inputs(wl: Workload, which=("x", "w", "dy")) -> dict:
    """CPU tensors in storage dtype: x [B,C,L] ~ N(0,1), w [C,K], dy [B,C,L] ~ N(0,1)."""
    out = {}
    shape = (wl.B, wl.C, wl.L)
    if "x" in which:
        out["x"] = torch.randn(shape, generator=_gen(BASE_SEED + wl.index), dtype=torch.float32).to(torch_dtype(wl)).contiguous()
    if "w" in which:
        out["w"] = make_filter(wl)
    if "dy" in which:
        out["dy"] = torch.randn(shape, generator=_gen(BASE_SEED + wl.index + 200), dtype=torch.float32).to(torch_dtype(wl)).contiguous()
    return out


def as_f32_numpy(t: torch.Tensor):
    """Exact widening of a storage-dtype CPU tensor to a float32 numpy array."""
    return t.detach().cpu().to(torch.float32).contiguous().numpy()
