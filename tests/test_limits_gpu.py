"""Edges of the contract in include/dwconv.h: tensors above 2^32 bytes (64-bit row offsets next to 32-bit
segment walks) and non-finite inputs (the matrix-core kernels multiply the zero taps of their edge Toeplitz blocks
and the zero-filled halos, where the definition of Sec. IV-A skips the term)."""
import numpy as np
import pytest
import torch

from paper_2604_25422_amd import binding
from paper_2604_25422_amd.workloads import as_f32_numpy

pytestmark = pytest.mark.gpu


def _device_ints(shape, seed, lim, tdt):
    """Seeded integers in [-lim, lim], drawn on the device batch by batch (the tensor is larger than 4 GiB)."""
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    out = torch.empty(shape, dtype=tdt, device="cuda")
    step = max(1, (1 << 28) // (shape[1] * shape[2]))
    for a in range(0, shape[0], step):
        n = min(step, shape[0] - a)
        out[a:a + n] = torch.randint(-lim, lim + 1, (n,) + tuple(shape[1:]), generator=g, dtype=torch.int8, device="cuda").to(tdt)
    return out


# (B, C, L, K, pad_left, storage, lim): x and dY are integers in [-lim, lim], w in [-3, 3]; every sum stays
# below 2^24, so the comparison with the oracle is exact.  Rows (fwd, dX) of the first, a middle and the last batch
# and the channels 0, C/2 and C-1 (dW, over all batches) are checked: the first and last bytes of the tensor, and
# element offsets on both sides of 2^31 and 2^32.
@pytest.mark.parametrize("B,C,L,K,p,dtype,lim", [
    (1100, 1024, 2048, 32, 31, "bf16", 2),       # 4.6 GB per tensor: register-resident filters, bf16 matrix instruction
    (600, 1024, 2048, 64, 63, "f32", 3),         # 5.0 GB per tensor: headline class, one workgroup per channel for dW
    (190000, 128, 48, 48, 24, "f32", 1),         # 4.7 GB per tensor: the paper's rows, sixteen to a matrix tile
    (50, 96, 300000, 7, 3, "f32", 1),            # 5.8 GB per tensor: rows of 1.2 MB, 293 segments each
])
def test_tensors_above_4_GiB(oracle_mod, B, C, L, K, p, dtype, lim):
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    es = 4 if dtype == "f32" else 2
    assert B * C * L * es > 1 << 32 and lim * lim * B * L < 1 << 24 and 3 * lim * K < 1 << 24
    print(f"case above 4 GiB {dtype} B{B} C{C} L{L} K{K} p{p}: {B * C * L * es / 2 ** 30:.2f} GiB per tensor", flush=True)
    x = _device_ints((B, C, L), 61, lim, tdt)
    dy = _device_ints((B, C, L), 62, lim, tdt)
    g = torch.Generator(device="cpu"); g.manual_seed(63)
    w = torch.randint(-3, 4, (C, K), generator=g, dtype=torch.int32).to(tdt)
    wd = w.cuda()
    y = binding.dwconv_fwd(x, wd, p)
    dx = binding.dwconv_bwd_input(dy, wd, p)
    dw = binding.dwconv_bwd_weight(x, dy, K, p)
    torch.cuda.synchronize()
    dx_f = torch.empty_like(dx)
    _, dw_f = binding.dwconv_bwd(dy, x, wd, p, out_dx=dx_f)
    torch.cuda.synchronize()
    assert torch.equal(dx_f, dx), "dwconv_bwd: dx differs from dwconv_bwd_input"
    del dx_f
    wn = as_f32_numpy(w)
    bsel = [0, B // 2, B - 1]
    xs = as_f32_numpy(x[bsel].cpu()); dys = as_f32_numpy(dy[bsel].cpu())
    ref, _ = oracle_mod.fwd(xs, wn, p)
    assert torch.equal(y[bsel].cpu(), torch.from_numpy(ref).float().to(tdt)), "fwd differs on the sampled batches"
    ref, _ = oracle_mod.bwd_input(dys, wn, p)
    assert torch.equal(dx[bsel].cpu(), torch.from_numpy(ref).float().to(tdt)), "dX differs on the sampled batches"
    csel = [0, C // 2, C - 1]
    xc = as_f32_numpy(x[:, csel].contiguous().cpu()); dyc = as_f32_numpy(dy[:, csel].contiguous().cpu())
    ref, _ = oracle_mod.bwd_weight(xc, dyc, K, p)
    assert np.all(np.abs(ref) < 2.0 ** 24)
    exp = torch.from_numpy(ref).float().to(tdt)
    assert torch.equal(dw[csel].cpu(), exp), "dW differs on the sampled channels"
    assert torch.equal(dw_f[csel].cpu(), exp), "dW of dwconv_bwd differs on the sampled channels"


# Non-finite inputs.  The contract (include/dwconv.h): an Inf or NaN at position u of row (b, c) reaches, besides the
# outputs the definition gives it, at most the outputs of the same row within 63 positions of those and the last 63
# positions of row (b - 1, c) / the first 63 of row (b + 1, c) (short rows of a channel are processed end to end); no
# other channel is touched.  In the weight gradient it may reach every coefficient of its channel and no other channel.
# (B, C, L, K, pad_left, storage): one shape per kernel family.
NONFINITE = [
    (2, 3, 2600, 64, 63, "f32"), (2, 3, 2600, 64, 20, "f32"), (2, 3, 2600, 7, 3, "f32"), (2, 3, 2600, 130, 129, "f32"),
    (2, 3, 2608, 64, 63, "bf16"), (2, 3, 2608, 200, 100, "bf16"),
    (40, 4, 48, 48, 24, "f32"), (40, 4, 48, 48, 24, "bf16"), (60, 4, 200, 31, 15, "f32"),
    (2, 3, 1024, 700, 699, "f32"), (2, 3, 1024, 700, 350, "bf16"),
    (2, 3, 1001, 9, 4, "f32"), (2, 3, 1001, 300, 299, "f32"),
]
SLOP = 63


@pytest.mark.parametrize("B,C,L,K,p,dtype", NONFINITE)
@pytest.mark.parametrize("bad", [float("inf"), float("nan")])
def test_non_finite_inputs_stay_where_the_contract_says(B, C, L, K, p, dtype, bad):
    print(f"case non-finite {bad} {dtype} B{B} C{C} L{L} K{K} p{p}", flush=True)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    g = torch.Generator(device="cpu"); g.manual_seed(77)
    x = torch.randn((B, C, L), generator=g).to(tdt); dy = torch.randn((B, C, L), generator=g).to(tdt)
    w = torch.randn((C, K), generator=g).to(tdt)
    w[w == 0] = 1.0
    b0, c0 = B - 1, 1
    for u in (0, L // 2 + 3, L - 1):
        xb = x.clone(); xb[b0, c0, u] = bad
        dyb = dy.clone(); dyb[b0, c0, u] = bad
        xd, xbd, dyd, dybd, wd = x.cuda(), xb.cuda(), dy.cuda(), dyb.cuda(), w.cuda()
        y0 = binding.dwconv_fwd(xd, wd, p); y1 = binding.dwconv_fwd(xbd, wd, p)
        d0 = binding.dwconv_bwd_input(dyd, wd, p); d1 = binding.dwconv_bwd_input(dybd, wd, p)
        g0 = binding.dwconv_bwd_weight(xd, dyd, K, p); g1 = binding.dwconv_bwd_weight(xbd, dyd, K, p)
        g2 = binding.dwconv_bwd_weight(xd, dybd, K, p)
        torch.cuda.synchronize()
        # fwd: x[u] enters y[t] for t = u - j + p, j = 0..K-1;  dX: dy[u] enters dx[s] for s = u + j - p
        for name, clean, dirty, lo, hi in (("fwd", y0, y1, u + p - K + 1, u + p), ("dx", d0, d1, u - p, u - p + K - 1)):
            lo_d, hi_d = max(lo, 0), min(hi, L - 1)
            same = torch.ones((B, C, L), dtype=torch.bool)
            same[b0, c0, max(lo - SLOP, 0):min(hi + SLOP, L - 1) + 1] = False
            same[b0 - 1, c0, max(L - SLOP, 0):] = False          # (b0 is the last batch: no row after it)
            assert torch.equal(clean.cpu()[same], dirty.cpu()[same]), f"{name}: position {u} reached outside its footprint"
            assert torch.isfinite(clean).all()
            assert not torch.isfinite(dirty[b0, c0, lo_d:hi_d + 1]).any(), f"{name}: position {u} must poison [{lo_d}, {hi_d}]"
        # dW: other channels keep their bits; the coefficients the definition reaches are not finite
        for name, dirty, jlo, jhi in (("dw (x)", g1, u + p - L + 1, u + p), ("dw (dy)", g2, p - u, p - u + L - 1)):
            other = [c for c in range(C) if c != c0]
            assert torch.equal(g0[other], dirty[other]), f"{name}: another channel changed"
            jl, jh = max(jlo, 0), min(jhi, K - 1)
            assert not torch.isfinite(dirty[c0, jl:jh + 1]).any(), f"{name}: coefficients [{jl}, {jh}] must not be finite"
