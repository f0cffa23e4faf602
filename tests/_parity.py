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


# max |gpu - oracle| / sum|terms| allowed per path
TOL = {("f32", "fwd"): 1e-5, ("f32", "dx"): 1e-5, ("f32", "dw"): 1e-4,
       ("bf16", "fwd"): 2e-2, ("bf16", "dx"): 2e-2, ("bf16", "dw"): 2e-2}


def seeded(shape, seed, dtype):
    g = torch.Generator(device="cpu"); g.manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32).to(dtype).contiguous()


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
