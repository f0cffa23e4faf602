"""The allocation-free weight-gradient entry point (dwconv_bwd_weight_noalloc): partial sums in the library's
built-in scratch instead of a caller's workspace.  It must give the bits of dwconv_bwd_weight (same kernels, same
order of sums) and meet the oracle's bound, on two calls in a row, the second on a smaller input that leaves most of
the scratch holding the first call's partial sums."""
import numpy as np
import pytest
import torch

from _parity import TOL, normalised_error, seeded
from paper_2604_25422_amd import binding
from paper_2604_25422_amd.workloads import as_f32_numpy

pytestmark = pytest.mark.gpu

# (B, C, L, K, pad_left): first a shape with several slices per coefficient, then a smaller one; a long filter
# (two zero-filled slices that even and odd offset groups add into) followed by a shorter long filter.
PAIRS = [
    ("f32", (50, 100, 5000, 40, 11), (7, 60, 3000, 20, 19)),
    ("bf16", (33, 130, 2048, 64, 63), (9, 70, 1032, 24, 3)),
    ("f32", (3, 20, 2048, 2048, 2047), (2, 12, 1024, 700, 350)),
    ("f32", (300, 96, 200, 31, 15), (37, 50, 48, 48, 24)),
]


def _one(oracle, dtype, shape, seed):
    B, C, L, K, p = shape
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = seeded((B, C, L), 4100 + seed, tdt)
    dy = seeded((B, C, L), 4200 + seed, tdt)
    xd, dyd = x.cuda(), dy.cuda()
    out = torch.full((C, K), float("nan"), dtype=tdt, device="cuda")
    got = binding.dwconv_bwd_weight_noalloc(xd, dyd, K, p, out=out)
    ref_call = binding.dwconv_bwd_weight(xd, dyd, K, p)
    torch.cuda.synchronize()
    assert torch.equal(got, ref_call), f"{dtype} {shape}: differs from dwconv_bwd_weight"
    r, ra = oracle.bwd_weight(as_f32_numpy(x), as_f32_numpy(dy), K, p)
    e, i = normalised_error(got.float().cpu().numpy(), r, ra)
    assert e <= TOL[(dtype, "dw")], (dtype, shape, e, i)
    return binding.dwconv_bwd_weight_slices(B, C, L, K, p, binding.F32 if dtype == "f32" else binding.BF16)


@pytest.mark.parametrize("dtype,first,second", PAIRS)
def test_noalloc_two_calls_in_a_row(oracle_mod, dtype, first, second):
    s1 = _one(oracle_mod, dtype, first, 1)
    s2 = _one(oracle_mod, dtype, second, 2)
    print(f"slices: {first} -> {s1}, {second} -> {s2}", flush=True)
    assert max(s1, s2) > 1, "at least one of the two shapes must go through the scratch"


def test_noalloc_rejects_what_does_not_fit():
    # two slices of 512 x 8192 fp32 coefficients = 32 MiB > the built-in 16 MiB
    B, C, L, K, p = 1, 512, 8192, 8192, 8191
    assert binding.dwconv_bwd_weight_workspace_bytes(B, C, L, K, p, binding.F32) > binding.dwconv_noalloc_scratch_bytes()
    x = torch.zeros((B, C, L), device="cuda"); dy = torch.zeros_like(x)
    out = torch.zeros((C, K), device="cuda")
    with pytest.raises(binding.DwconvError) as ei:
        binding.dwconv_bwd_weight_noalloc(x, dy, K, p, out=out)
    assert ei.value.status == 8
    assert "scratch" in str(ei.value)
