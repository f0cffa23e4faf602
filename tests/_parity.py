"""Helpers of the GPU parity tests: run the HIP path through the C ABI binding and the
fp64 CPU oracle on the same seeded inputs and return the normalised errors."""
import numpy as np
import torch

from paper_2604_25422_amd import binding
from paper_2604_25422_amd.workloads import as_f32_numpy

def normalised_error(got, ref, ref_abs, floor=2.0 ** -100):
    """max_i |got_i - ref_i| / max(sum_i|terms|, floor).  Returns (err, argmax)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.maximum(np.asarray(ref_abs, dtype=np.float64), floor)
    e = np.abs(got - ref) / den
    if not np.all(np.isfinite(got)):
        return float("inf"), int(np.argmin(np.isfinite(got).ravel()))
    i = int(np.argmax(e))
    return float(e.ravel()[i]), i


def normalised_error_rows(got, ref, ref_abs, floor=2.0 ** -100):
    """normalised_error over the leading axis in slabs (same value; bounded temporaries for 1e8-element tensors)."""
    worst, at = 0.0, 0
    n = got.shape[0]
    per = int(np.prod(got.shape[1:]))
    step = max(1, (1 << 24) // max(per, 1))
    for a in range(0, n, step):
        e, i = normalised_error(got[a:a + step], ref[a:a + step], ref_abs[a:a + step], floor)
        if e > worst or not np.isfinite(e):
            worst, at = e, a * per + i
        if not np.isfinite(e):
            break
    return worst, at


# max |gpu - oracle| / sum|terms| allowed per path
TOL = {("f32", "fwd"): 1e-5, ("f32", "dx"): 1e-5, ("f32", "dw"): 1e-4,
       ("bf16", "fwd"): 2e-2, ("bf16", "dx"): 2e-2, ("bf16", "dw"): 2e-2}


def seeded(shape, seed, dtype):
    g = torch.Generator(device="cpu"); g.manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32).to(dtype).contiguous()


def small_ints(shape, seed, lim, dtype):
    """Seeded integers in [-lim, lim] (exact in fp32 and bf16 for lim <= 256): every product and every partial sum
    of the operator is then an integer, exact in fp32 up to 2^24 whatever the order of summation."""
    g = torch.Generator(device="cpu"); g.manual_seed(seed)
    return torch.randint(-lim, lim + 1, shape, generator=g, dtype=torch.int32).to(dtype).contiguous()


def to_device(t, offset=0):
    """A device copy of t; with offset > 0 a view that starts `offset` elements into a larger allocation, so that
    its base pointer is aligned to the element size only."""
    if offset == 0:
        return t.cuda()
    buf = torch.empty(t.numel() + offset + 8, dtype=t.dtype, device="cuda")
    v = buf[offset:offset + t.numel()].view(t.shape)
    v.copy_(t)
    return v


def empty_device(shape, dtype, offset=0):
    n = int(np.prod(shape))
    buf = torch.empty(n + offset + 8, dtype=dtype, device="cuda")
    return buf[offset:offset + n].view(shape)


def gpu_all(x, w, dy, p):
    """fwd, dX, dW through the C ABI; returns float64 numpy arrays (outputs widened exactly)."""
    xd, wd, dyd = x.cuda(), w.cuda(), dy.cuda()
    K = w.shape[1]
    y = binding.dwconv_fwd(xd, wd, p)
    dx = binding.dwconv_bwd_input(dyd, wd, p)
    dw = binding.dwconv_bwd_weight(xd, dyd, K, p)
    torch.cuda.synchronize()
    return tuple(t.float().cpu().numpy().astype(np.float64) for t in (y, dx, dw))


def oracle_all(oracle, x, w, dy, p):
    xn, wn, dyn = as_f32_numpy(x), as_f32_numpy(w), as_f32_numpy(dy)
    K = wn.shape[1]
    return oracle.fwd(xn, wn, p), oracle.bwd_input(dyn, wn, p), oracle.bwd_weight(xn, dyn, K, p)


def check_case(oracle, B, C, L, K, p, dtype="f32", seed=0):
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = seeded((B, C, L), 1000 + seed, tdt)
    w = seeded((C, K), 2000 + seed, tdt)
    dy = seeded((B, C, L), 3000 + seed, tdt)
    got = gpu_all(x, w, dy, p)
    ref = oracle_all(oracle, x, w, dy, p)
    errs = {}
    for name, g, (r, ra) in zip(("fwd", "dx", "dw"), got, ref):
        e, i = normalised_error(g, r, ra)
        errs[name] = e
        assert e <= TOL[(dtype, name)], (
            f"{name} B{B} C{C} L{L} K{K} p{p} {dtype}: err {e:.3e} > {TOL[(dtype, name)]:.0e} at flat index {i}: "
            f"gpu {g.ravel()[i]!r} oracle {r.ravel()[i]!r}")
        # outputs whose index set is empty must be exactly zero
        empty = (ra == 0)
        assert np.all(g[empty] == 0), f"{name}: non-zero output where no term exists"
    return errs
