"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.
Where the oracle cannot finish the whole tensor in seconds, sampled rows (fwd, dX) and
sampled channels (dW) are checked one by one: rows and channels are independent, so the
oracle evaluates exactly the sampled outputs of the full-size problem."""
import numpy as np
import pytest
import torch

from _parity import TOL
from paper_2604_25422_amd import binding, workloads
from _parity import normalised_error
from paper_2604_25422_amd.workloads import as_f32_numpy

pytestmark = pytest.mark.gpu


def run_full_size(oracle, wl, n_rows, n_chans, seed=0):
    inp = workloads.make_inputs(wl)
    x, w, dy = inp["x"], inp["w"], inp["dy"]
    xd, wd, dyd = x.cuda(), w.cuda(), dy.cuda()
    y = binding.dwconv_fwd(xd, wd, wl.pad_left)
    dx = binding.dwconv_bwd_input(dyd, wd, wl.pad_left)
    dw = binding.dwconv_bwd_weight(xd, dyd, wl.K, wl.pad_left)
    dw2 = binding.dwconv_bwd_weight(xd, dyd, wl.K, wl.pad_left)
    torch.cuda.synchronize()
    assert torch.equal(dw, dw2), "weight gradient must be bitwise reproducible"
    # the fused backward call at the same size: same dx bits, dw checked below like the separate one
    dx_f, dw_f = binding.dwconv_bwd(dyd, xd, wd, wl.pad_left)
    torch.cuda.synchronize()
    assert torch.equal(dx_f, dx), "fused backward: dx differs from the separate path"
    dw_f = dw_f.float().cpu()
    del dx_f
    y, dx, dw = y.float().cpu(), dx.float().cpu(), dw.float().cpu()
    del xd, dyd
    rng = np.random.default_rng(seed)
    rows = B_C = wl.B * wl.C
    n_rows = min(n_rows, rows); n_chans = min(n_chans, wl.C)
    # always include the first and last row / channel
    rsel = np.unique(np.concatenate([[0, rows - 1], rng.choice(rows, n_rows, replace=False)]))
    csel = np.unique(np.concatenate([[0, wl.C - 1], rng.choice(wl.C, n_chans, replace=False)]))
    xf = as_f32_numpy(x).reshape(rows, wl.L); dyf = as_f32_numpy(dy).reshape(rows, wl.L); wf = as_f32_numpy(w)
    errs = {}
    # sampled rows: a [1, R, L] problem whose channel r carries the filter of the sampled row's channel
    xr = np.ascontiguousarray(xf[rsel])[None]; dyr = np.ascontiguousarray(dyf[rsel])[None]
    wr = np.ascontiguousarray(wf[rsel % wl.C])
    r, ra = oracle.fwd(xr, wr, wl.pad_left)
    errs["fwd"], _ = normalised_error(y.reshape(rows, wl.L).numpy()[rsel][None], r, ra)
    r, ra = oracle.bwd_input(dyr, wr, wl.pad_left)
    errs["dx"], _ = normalised_error(dx.reshape(rows, wl.L).numpy()[rsel][None], r, ra)
    # sampled channels, all batches and positions
    xc = np.ascontiguousarray(xf.reshape(wl.B, wl.C, wl.L)[:, csel]); dyc = np.ascontiguousarray(dyf.reshape(wl.B, wl.C, wl.L)[:, csel])
    r, ra = oracle.bwd_weight(xc, dyc, wl.K, wl.pad_left)
    errs["dw"], _ = normalised_error(dw.numpy()[csel], r, ra)
    errs["dw_fused"], _ = normalised_error(dw_f.numpy()[csel], r, ra)
    print(wl.name, {k: f"{v:.2e}" for k, v in errs.items()}, f"rows {len(rsel)} chans {len(csel)}", flush=True)
    for k, v in errs.items():
        assert v <= TOL[(wl.dtype, k.split("_")[0])], (wl.name, k, v)
    return errs


def test_cfg0_small_whole(oracle_mod):
    run_full_size(oracle_mod, workloads.WORKLOADS[0], 10 ** 9, 10 ** 9)


def test_cfg1_headline_full_size(oracle_mod):
    run_full_size(oracle_mod, workloads.WORKLOADS[1], 1024, 32)


def test_cfg2_short_filter_full_size(oracle_mod):
    run_full_size(oracle_mod, workloads.WORKLOADS[2], 4096, 64)


def test_cfg3_long_filter_full_size(oracle_mod):
    run_full_size(oracle_mod, workloads.WORKLOADS[3], 48, 6)


def test_cfg4_bf16_full_size(oracle_mod):
    run_full_size(oracle_mod, workloads.WORKLOADS[4], 4096, 48)


def test_paper_shape_full_size(oracle_mod):
    # the shape the paper measures (Sec. V): many short rows, sixteen rows to a matrix tile
    run_full_size(oracle_mod, workloads.WORKLOADS[5], 8192, 16)


def test_mid_filter_full_size(oracle_mod):
    # a filter of 128 taps at the headline geometry: nine block offsets on the register-resident kernels
    run_full_size(oracle_mod, workloads.WORKLOADS[6], 512, 16)


def test_long_filter_bf16_full_size(oracle_mod):
    # the long-filter configuration on bf16 storage: the bf16 matrix-instruction long-filter kernels
    run_full_size(oracle_mod, workloads.WORKLOADS[8], 48, 6)


def test_mid_filter_bf16_full_size(oracle_mod):
    # the same 128 taps on bf16 storage: nine block offsets on the bf16 matrix-instruction kernels
    run_full_size(oracle_mod, workloads.WORKLOADS[7], 512, 16)


@pytest.mark.parametrize("B,C,L,K,p,dtype", [
    (50, 100, 5000, 40, 11, "f32"),        # channel count unrelated to the chip, ragged last segment, several slices
    (7, 300, 12000, 64, 63, "f32"),        # long rows, odd batch
    (33, 257, 2040, 20, 19, "bf16"),       # bf16, odd channel count, row length a multiple of 8 but not of 16
    (600, 96, 200, 31, 15, "f32"),         # short rows: virtual rows with several slices
    (600, 96, 200, 31, 15, "bf16"),        # the same on bf16 storage (widening kernels)
    (8192, 128, 48, 48, 24, "bf16"),       # half the paper's batch on bf16 storage: sixteen rows per tile, channel pairs
    (5000, 130, 64, 64, 63, "f32"),        # rows of four blocks, six block offsets, batch not a multiple of sixteen
    (24, 256, 4096, 128, 127, "f32"),      # nine block offsets (fp32 filters up to 130 taps)
])
def test_mid_size_odd_shapes(oracle_mod, B, C, L, K, p, dtype):
    wl = workloads.Workload(f"odd_B{B}_C{C}_L{L}_K{K}_p{p}_{dtype}", 9, B, C, L, K, p, dtype, "normal")
    run_full_size(oracle_mod, wl, 512, 12)
