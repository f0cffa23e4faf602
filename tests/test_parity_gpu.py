"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the
same seeded inputs.  Tolerances: max |gpu - oracle| / sum|terms| <= 1e-5 (fp32 fwd, dX),
1e-4 (fp32 dW), 2e-2 (bf16 storage)."""
import os

import numpy as np
import pytest
import torch

from _parity import TOL, check_case, gpu_all, oracle_all, seeded

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2604_25422_amd import binding
    binding.lib()


# (B, C, L, K, pad_left): ragged tails, L not a multiple of 4/16/64, K = 1, K > L, every pad class
SMALL = [
    (1, 1, 1, 1, 0), (1, 1, 5, 3, 1), (2, 3, 7, 4, 2), (1, 2, 4, 6, 5), (3, 2, 33, 1, 0),
    (2, 3, 100, 5, 0), (2, 3, 100, 5, 2), (2, 3, 100, 5, 4),
    (2, 5, 257, 7, 3), (1, 4, 1023, 16, 15), (2, 4, 1025, 16, 8), (1, 3, 2050, 9, 4),
    (3, 7, 333, 31, 30), (2, 2, 48, 48, 24), (2, 2, 48, 48, 47), (5, 3, 48, 48, 0),
    (1, 2, 40, 100, 99), (1, 2, 40, 100, 50), (2, 2, 130, 260, 129),
    (2, 3, 600, 64, 63), (1, 2, 4100, 64, 32), (2, 2, 1500, 300, 299), (1, 1, 3000, 700, 350),
    (1, 2, 1100, 1030, 1029),
    # long-filter matrix-core kernels: odd batch (row pairing), paper-style and anti-causal pads, every group size
    (3, 2, 256, 200, 100), (2, 3, 512, 512, 511), (1, 2, 2048, 1500, 700), (2, 2, 1024, 130, 129),
    (1, 1, 1024, 90, 0), (3, 1, 640, 640, 320), (1, 2, 4096, 4096, 4095), (2, 1, 1000, 2500, 1200),
    (1, 1, 8192, 300, 299), (1, 2, 72, 67, 66),
    # seven to ten block offsets (fp32 register-resident class up to K = 130): every count, ragged rows, several rows per wave
    (3, 5, 2060, 100, 99), (2, 3, 1028, 112, 50), (5, 2, 3072, 128, 127), (2, 2, 1100, 130, 0), (9, 4, 1024, 97, 96),
    # eleven to sixteen block offsets: register-resident kernels (fwd/dX: rows that fill three quarters of their
    # 1024-position segments, the long-filter kernel otherwise); every count, ragged rows, several segments per wave
    (3, 4, 2060, 160, 159), (2, 3, 1028, 226, 100), (5, 2, 3072, 200, 0), (2, 2, 1100, 180, 90),
    (7, 2, 1024, 161, 80), (3, 3, 1024, 176, 175), (2, 5, 800, 190, 95), (4, 2, 3000, 215, 214), (2, 3, 2048, 226, 225),
    (2, 2, 4092, 226, 0), (70, 32, 1024, 170, 169),
    # seventeen to thirty-two block offsets: the weight gradient in two passes over the offsets (second pass with
    # windows that start past the end of the row when pad is small), fwd/dX on the long-filter kernel
    (3, 4, 1024, 256, 255), (2, 3, 2048, 300, 150), (2, 2, 3000, 482, 481), (5, 2, 1024, 400, 0), (4, 2, 4092, 350, 100),
    (70, 32, 1024, 260, 259), (1, 1, 800, 480, 0),
    # long filters on short rows: many rows per workgroup, batches that are not whole groups of them
    (21, 2, 1024, 600, 599), (11, 2, 2048, 900, 450), (37, 1, 512, 700, 0),
    # thirty-three to forty-eight block offsets: the weight gradient in three passes
    (2, 3, 2048, 700, 350), (2, 2, 3000, 513, 0), (40, 8, 1024, 530, 529), (3, 2, 1024, 738, 737),
    # filters or rows beyond 8192: tiled long-filter forward / input gradient, many-launch weight gradient
    (1, 2, 9000, 300, 299), (1, 1, 16384, 16384, 16383), (2, 1, 12000, 9000, 4000), (3, 1, 8200, 8200, 0),
    (1, 2, 9000, 900, 899), (1, 1, 32768, 20000, 19999),
    # matrix-core kernels at row lengths that are multiples of 4 but not of 8, 16 or 64
    (2, 3, 1004, 32, 31), (3, 2, 36, 16, 15), (2, 2, 2060, 64, 63), (1, 5, 44, 7, 3),
]


# Rows of at most 64 positions (fp32, L % 4 == 0): sixteen rows of a channel per matrix tile.  Batches that are
# not whole units of sixteen, rows that are not whole 16-blocks, every number of block offsets, every pad class,
# many units per wave, channel counts that give whole-channel workgroups.
SHORT_ROWS = [
    (1, 1, 4, 3, 1), (16, 2, 16, 3, 0), (17, 3, 16, 16, 15), (15, 2, 20, 5, 2), (33, 3, 32, 16, 8),
    (31, 2, 36, 31, 30), (40, 5, 48, 48, 24), (64, 2, 48, 48, 47), (100, 3, 48, 48, 0), (7, 4, 52, 20, 10),
    (50, 2, 64, 64, 63), (48, 3, 64, 66, 33), (129, 2, 60, 40, 0), (300, 9, 48, 48, 24), (1000, 2, 12, 7, 3),
    (2100, 1, 48, 33, 16), (70, 256, 48, 48, 24), (36, 512, 24, 9, 4), (20, 2, 8, 50, 25),
    # rows of five to eight blocks (weight-gradient units of four rows)
    (40, 3, 68, 7, 3), (33, 2, 80, 48, 24), (17, 5, 96, 64, 63), (9, 4, 100, 66, 0), (130, 2, 128, 31, 15),
    (50, 256, 128, 16, 15), (21, 3, 124, 33, 32), (6, 2, 112, 5, 2),
]


@pytest.mark.parametrize("B,C,L,K,p", SHORT_ROWS)
def test_short_rows_f32(oracle_mod, B, C, L, K, p):
    print(f"case short rows f32 B{B} C{C} L{L} K{K} p{p}", flush=True)
    check_case(oracle_mod, B, C, L, K, p, "f32", seed=B + C + L + K)


# the same kernels on bf16 storage (rows widened to fp32 on the way into LDS, one rounding at the store)
@pytest.mark.parametrize("B,C,L,K,p", SHORT_ROWS)
def test_short_rows_bf16(oracle_mod, B, C, L, K, p):
    print(f"case short rows bf16 B{B} C{C} L{L} K{K} p{p}", flush=True)
    check_case(oracle_mod, B, C, L, K, p, "bf16", seed=B + C + L + K + 1)


# Rows of a million positions and more: byte offsets inside a row beyond 2^22, thousands of segments per row.
@pytest.mark.parametrize("B,C,L,K,p,dtype", [
    (1, 2, (1 << 20) + 4, 64, 63, "f32"), (1, 1, 3000004, 7, 3, "f32"), (1, 2, (1 << 20) + 8, 32, 31, "bf16"),
    (1, 1, (1 << 21) + 12, 100, 50, "f32"),
])
def test_long_rows(oracle_mod, B, C, L, K, p, dtype):
    print(f"case long rows {dtype} B{B} C{C} L{L} K{K} p{p}", flush=True)
    check_case(oracle_mod, B, C, L, K, p, dtype, seed=5)


@pytest.mark.parametrize("B,C,L,K,p", SMALL)
def test_small_shapes_f32(oracle_mod, B, C, L, K, p):
    print(f"case f32 B{B} C{C} L{L} K{K} p{p}", flush=True)
    check_case(oracle_mod, B, C, L, K, p, "f32", seed=B + C + L + K)


@pytest.mark.parametrize("B,C,L,K,p", SMALL[::2] + [(4, 6, 1024, 32, 31), (3, 5, 1000, 32, 16), (2, 3, 1004, 32, 31),
                                                   (3, 2, 256, 200, 100), (1, 2, 2048, 1500, 700), (2, 2, 2056, 64, 0),
                                                   # bf16 short rows longer than 64 positions: virtual rows
                                                   (40, 6, 128, 16, 15), (33, 3, 100, 31, 30), (9, 256, 256, 33, 16),
                                                   (64, 2, 512, 64, 63), (7, 5, 68, 7, 3), (300, 2, 72, 48, 24),
                                                   # bf16 forward / dX with seven to sixteen block offsets: every count
                                                   (3, 5, 2048, 100, 99), (2, 3, 1024, 112, 50), (5, 2, 3072, 128, 127),
                                                   (9, 4, 1024, 130, 0), (7, 2, 1024, 161, 80), (3, 3, 1024, 176, 175),
                                                   (2, 5, 800, 190, 95), (4, 2, 3000, 215, 214), (2, 3, 2048, 226, 225),
                                                   (2, 2, 4088, 200, 0), (70, 32, 1024, 170, 169), (2, 3, 1028, 150, 149),
                                                   # bf16 long filters (forward / dX on the bf16 matrix instruction): odd
                                                   # batches, every pad class, filters longer than the row, ragged rows
                                                   (2, 3, 512, 512, 511), (3, 1, 640, 640, 320), (1, 2, 4096, 4096, 4095),
                                                   (2, 1, 1000, 2500, 1200), (1, 1, 8192, 300, 299), (3, 2, 1024, 1024, 0),
                                                   (5, 2, 4100, 700, 350), (3, 3, 260, 513, 17), (1, 1, 8192, 8192, 8191),
                                                   # bf16 weight gradient in two passes over seventeen to thirty-two offsets
                                                   (3, 4, 1024, 256, 255), (2, 3, 2048, 300, 150), (2, 2, 3000, 482, 481),
                                                   (5, 2, 1024, 400, 0), (70, 32, 1024, 260, 259), (1, 1, 8192, 300, 299),
                                                   # long filters on short rows: many rows per workgroup, batches that
                                                   # are not whole groups of them
                                                   (21, 2, 1024, 600, 599), (11, 2, 2048, 900, 450), (37, 1, 512, 700, 0),
                                                   # bf16 weight gradient in three and four passes (33 to 64 offsets)
                                                   (2, 3, 2048, 700, 350), (3, 2, 1024, 994, 993), (2, 2, 3000, 513, 0),
                                                   (40, 8, 1024, 530, 529)])
def test_small_shapes_bf16(oracle_mod, B, C, L, K, p):
    print(f"case bf16 B{B} C{C} L{L} K{K} p{p}", flush=True)
    check_case(oracle_mod, B, C, L, K, p, "bf16", seed=B + C + L + K)


@pytest.mark.parametrize("B,C,L,K,p,dtype", [
    (4, 64, 1024, 16, 15, "f32"),          # configuration 0, whole
    (4, 16, 4096, 64, 63, "f32"),          # headline geometry, fewer rows
    (8, 32, 2048, 7, 3, "f32"),            # short-filter geometry
    (16, 24, 1024, 32, 31, "bf16"),        # bf16 geometry
    (2, 4, 2048, 2048, 2047, "f32"),       # filter as long as the sequence
])
def test_config_geometries_reduced(oracle_mod, B, C, L, K, p, dtype):
    print(f"case {dtype} B{B} C{C} L{L} K{K} p{p}", flush=True)
    check_case(oracle_mod, B, C, L, K, p, dtype, seed=7)


def test_weight_gradient_is_run_to_run_deterministic_and_two_stage_matches():
    from paper_2604_25422_amd import binding
    B, C, L, K, p = 6, 10, 3000, 48, 24
    x = seeded((B, C, L), 1, torch.float32).cuda(); dy = seeded((B, C, L), 2, torch.float32).cuda()
    a = binding.dwconv_bwd_weight(x, dy, K, p)
    b = binding.dwconv_bwd_weight(x, dy, K, p)
    ws = binding.dwconv_bwd_weight_partial(x, dy, K, p)
    c = binding.dwconv_bwd_weight_finalize(ws, B, C, L, K, p, torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(a, c)
    S = binding.dwconv_bwd_weight_slices(B, C, L, K, p, binding.F32)
    part = ws.view(torch.float32)[: S * C * K].view(S, C, K)
    seq = torch.zeros(C, K, device="cuda")
    for s in range(S):
        seq = seq + part[s]
    assert torch.equal(seq, a)             # stage 2 is the ordered sum of the stage-1 slices


def test_inputs_are_not_written_and_outputs_are_overwritten():
    from paper_2604_25422_amd import binding
    B, C, L, K, p = 2, 3, 500, 9, 4
    x = seeded((B, C, L), 3, torch.float32).cuda(); w = seeded((C, K), 4, torch.float32).cuda()
    x0, w0 = x.clone(), w.clone()
    y = torch.full_like(x, float("nan"))
    binding.dwconv_fwd(x, w, p, out=y)
    dx = torch.full_like(x, float("nan"))
    binding.dwconv_bwd_input(x, w, p, out=dx)
    dw = torch.full((C, K), float("nan"), device="cuda")
    ws = binding.new_workspace(x, K, p); ws.fill_(0xFF)
    binding.dwconv_bwd_weight(x, x, K, p, workspace=ws, out=dw)
    torch.cuda.synchronize()
    assert torch.equal(x, x0) and torch.equal(w, w0)
    assert torch.isfinite(y).all() and torch.isfinite(dx).all() and torch.isfinite(dw).all()


def test_runs_on_a_non_default_stream(oracle_mod):
    from paper_2604_25422_amd import binding
    from _parity import normalised_error
    B, C, L, K, p = 2, 4, 777, 12, 11
    x = seeded((B, C, L), 5, torch.float32); w = seeded((C, K), 6, torch.float32)
    st = torch.cuda.Stream()
    xd, wd = x.cuda(), w.cuda()
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        y = binding.dwconv_fwd(xd, wd, p)
    st.synchronize()
    r, ra = oracle_mod.fwd(x.numpy(), w.numpy(), p)
    e, _ = normalised_error(y.cpu().numpy(), r, ra)
    assert e <= 1e-5


# One workgroup per channel (C = 256, 512, 768 with enough segments per wave): the weight gradient is a single
# kernel that writes dw itself.  Ragged last segments, rows of one segment, fp32 and bf16.
SINGLE = [
    (8, 256, 4096, 16, 15, "f32"), (9, 256, 3900, 64, 63, "f32"), (33, 256, 1000, 33, 16, "f32"),
    (4, 512, 4096, 7, 3, "f32"), (17, 512, 1028, 48, 24, "f32"), (9, 512, 2048, 100, 99, "f32"), (20, 512, 1024, 128, 127, "f32"),
    (10, 768, 1024, 32, 31, "bf16"), (11, 768, 1032, 20, 0, "f32"), (40, 256, 1024, 64, 63, "bf16"),
]


@pytest.mark.parametrize("B,C,L,K,p,dtype", SINGLE)
def test_single_kernel_weight_gradient(oracle_mod, B, C, L, K, p, dtype):
    from paper_2604_25422_amd import binding
    print(f"case single {dtype} B{B} C{C} L{L} K{K} p{p}", flush=True)
    code = binding.F32 if dtype == "f32" else binding.BF16
    assert binding.dwconv_bwd_weight_single_pass(B, C, L, K, p, code)
    check_case(oracle_mod, B, C, L, K, p, dtype, seed=11)
    # the two-stage entry points give the same bits (one slice, copied by stage 2)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = seeded((B, C, L), 1011, tdt).cuda(); dy = seeded((B, C, L), 3011, tdt).cuda()
    one = binding.dwconv_bwd_weight(x, dy, K, p)
    ws = binding.dwconv_bwd_weight_partial(x, dy, K, p)
    two = binding.dwconv_bwd_weight_finalize(ws, B, C, L, K, p, tdt)
    again = binding.dwconv_bwd_weight(x, dy, K, p)
    torch.cuda.synchronize()
    assert torch.equal(one, two) and torch.equal(one, again)


# Fused backward call: dx and dw from one pass over dy (fp32, register-resident filters), the two separate paths
# for everything else.  (B, C, L, K, pad_left, dtype, fused?)
BWD = [
    (2, 3, 600, 64, 63, "f32", True), (1, 2, 4100, 64, 32, "f32", True), (3, 7, 336, 31, 30, "f32", True),
    (2, 3, 100, 5, 0, "f32", False), (2, 3, 100, 5, 4, "f32", False), (1, 4, 1024, 16, 15, "f32", True),
    (2, 4, 1028, 16, 8, "f32", True), (2, 2, 48, 48, 24, "f32", False), (5, 3, 48, 48, 0, "f32", False),
    (2, 2, 2060, 64, 63, "f32", True), (1, 5, 44, 7, 3, "f32", True), (20, 5, 68, 7, 3, "f32", False), (100, 6, 48, 48, 24, "f32", True), (37, 3, 64, 66, 33, "f32", False),
    (70, 256, 48, 48, 24, "f32", True), (300, 4, 20, 9, 8, "f32", True), (4, 16, 4096, 64, 63, "f32", True),
    (3, 2, 2048, 66, 65, "f32", True), (2, 2, 3072, 66, 0, "f32", True), (2, 3, 2052, 40, 20, "f32", True),
    (9, 256, 3900, 64, 63, "f32", True), (4, 512, 4096, 7, 3, "f32", True), (11, 768, 1032, 20, 0, "f32", True),
    (2, 5, 257, 7, 3, "f32", True), (2, 2, 1500, 300, 299, "f32", False), (3, 5, 1000, 32, 16, "bf16", True), (3, 5, 1004, 32, 16, "bf16", True), (3, 5, 1006, 32, 16, "bf16", True), (3, 5, 1007, 32, 16, "bf16", False),
    (2, 3, 2050, 64, 63, "f32", True), (3, 2, 1025, 7, 3, "f32", True), (2, 2, 4099, 48, 24, "f32", True), (2, 2, 770, 31, 0, "f32", True),
    (2, 2, 766, 31, 0, "f32", True),
    (4, 6, 1024, 32, 31, "bf16", True), (2, 3, 2056, 64, 0, "bf16", True), (10, 768, 1024, 32, 31, "bf16", True),
    (2, 2, 48, 48, 24, "bf16", False), (3, 2, 4096, 66, 65, "bf16", True), (40, 256, 1024, 64, 63, "bf16", True),
    (100, 6, 44, 31, 15, "bf16", True), (37, 3, 60, 20, 10, "bf16", False), (70, 256, 48, 48, 24, "bf16", True),
    (20, 4, 128, 16, 15, "bf16", True), (20, 4, 128, 16, 15, "f32", False), (20, 4, 132, 16, 15, "f32", True),
    (1, 2, 40, 100, 99, "f32", False), (3, 2, 33, 1, 0, "f32", False), (100, 6, 48, 200, 100, "f32", True), (40, 3, 96, 96, 48, "f32", False),
    (60, 4, 44, 500, 499, "bf16", True),
    # bf16 virtual rows: fused when rows start on a dword (even length)
    (40, 6, 200, 48, 24, "bf16", True), (30, 5, 196, 33, 16, "bf16", True), (7, 3, 520, 66, 65, "bf16", True),
    (64, 8, 136, 20, 19, "bf16", True), (600, 16, 200, 48, 47, "bf16", True), (25, 3, 264, 7, 3, "bf16", True),
    # ... from 64 positions (below: sixteen rows per tile, fused up to 48 positions only)
    (90, 5, 64, 48, 24, "bf16", True), (70, 6, 96, 33, 32, "bf16", True), (50, 3, 56, 16, 15, "bf16", False),
    (50, 3, 68, 16, 15, "bf16", True), (50, 3, 120, 66, 0, "bf16", True), (50, 3, 66, 16, 15, "bf16", True), (50, 3, 62, 16, 15, "bf16", False), (70, 4, 126, 48, 24, "bf16", True),
    (900, 16, 196, 48, 24, "bf16", True), (300, 8, 500, 64, 63, "bf16", True), (40, 4, 100, 7, 3, "bf16", True),
    # ... and of any even length from 129 positions (a row then ends two, four or six elements into a 16-byte granule)
    (40, 6, 198, 48, 24, "bf16", True), (30, 5, 250, 33, 16, "bf16", True), (25, 3, 130, 7, 3, "bf16", True),
    (700, 16, 202, 48, 47, "bf16", True), (30, 5, 199, 33, 16, "bf16", False),
    # fp32 virtual rows of any length (a row then ends one, two or three floats into a 16-byte granule)
    (40, 6, 198, 48, 24, "f32", True), (30, 5, 199, 33, 16, "f32", True), (25, 3, 133, 7, 3, "f32", True),
    (700, 16, 201, 48, 47, "f32", True), (300, 8, 365, 64, 63, "f32", True), (9, 4, 131, 100, 50, "f32", False),
]


@pytest.mark.parametrize("B,C,L,K,p,dtype,fused", BWD)
def test_fused_backward(oracle_mod, B, C, L, K, p, dtype, fused):
    from paper_2604_25422_amd import binding
    from _parity import normalised_error
    from paper_2604_25422_amd.workloads import as_f32_numpy
    print(f"case bwd {dtype} B{B} C{C} L{L} K{K} p{p}", flush=True)
    code = binding.F32 if dtype == "f32" else binding.BF16
    assert binding.dwconv_bwd_is_fused(B, C, L, K, p, code) == fused
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = seeded((B, C, L), 1021, tdt); w = seeded((C, K), 2021, tdt); dy = seeded((B, C, L), 3021, tdt)
    xd, wd, dyd = x.cuda(), w.cuda(), dy.cuda()
    dx, dw = binding.dwconv_bwd(dyd, xd, wd, p)
    dx_sep = binding.dwconv_bwd_input(dyd, wd, p)
    dx2, dw2 = binding.dwconv_bwd(dyd, xd, wd, p)
    torch.cuda.synchronize()
    assert torch.equal(dx, dx_sep), "fused dx differs from the separate input-gradient path"
    assert torch.equal(dx, dx2) and torch.equal(dw, dw2), "not run-to-run identical"
    xn, wn, dyn = as_f32_numpy(x), as_f32_numpy(w), as_f32_numpy(dy)
    for name, got, (ref, ra) in (("dx", dx, oracle_mod.bwd_input(dyn, wn, p)), ("dw", dw, oracle_mod.bwd_weight(xn, dyn, K, p))):
        g = got.float().cpu().numpy().astype(np.float64)
        e, i = normalised_error(g, ref, ra)
        assert e <= TOL[(dtype, name)], f"{name}: err {e:.3e} at flat index {i}: gpu {g.ravel()[i]!r} oracle {ref.ravel()[i]!r}"
        assert np.all(g[ra == 0] == 0)


def _random_shapes(n, seed):
    """Seeded shapes that mix every dispatch class: register-resident and long filters, short rows, rows that
    are not a multiple of 4, channel counts that trigger whole-channel workgroups, every pad class."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        K = int(rng.choice([1, 2, 3, 5, 7, 16, 31, 32, 33, 48, 64, 66, 67, 90, 100, 128, 130, 160, 200, 226, 227, 300, 513, 738, 739, 1000]))
        L = int(rng.choice([4, 12, 20, 36, 48, 52, 64, 68, 100, 128, 257, 512, 770, 1000, 1024, 1026, 1027, 1028, 2048, 2049, 2050, 3000,
                            3001, 4096, 4098]))
        C = int(rng.choice([1, 2, 3, 5, 8, 16, 256, 512]))
        B = int(rng.choice([1, 2, 3, 7, 16, 17, 40, 130]))
        if C >= 256:
            L = min(L, 128); B = int(rng.choice([8, 64, 300]))
        if B * C * L * min(K, L) > 6e7 or B * C * L > 4e6:
            continue
        p = int(rng.choice([0, K // 2, K - 1, int(rng.integers(0, K))]))
        dtype = "bf16" if rng.random() < 0.3 else "f32"
        out.append((B, C, L, K, p, dtype))
    return out


# DWCONV_SWEEP_N / DWCONV_SWEEP_SEED widen or move the sweep for a one-off soak; the defaults are what the suite runs.
@pytest.mark.parametrize("B,C,L,K,p,dtype", _random_shapes(int(os.environ.get("DWCONV_SWEEP_N", "180")),
                                                           int(os.environ.get("DWCONV_SWEEP_SEED", "20260425"))))
def test_random_shapes(oracle_mod, B, C, L, K, p, dtype):
    from paper_2604_25422_amd import binding
    print(f"case random {dtype} B{B} C{C} L{L} K{K} p{p}", flush=True)
    check_case(oracle_mod, B, C, L, K, p, dtype, seed=B + 3 * C + 5 * L + 7 * K + p)
    # the fused backward call on the same inputs: same dx bits as the separate call, dw within tolerance
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    sd = B + 3 * C + 5 * L + 7 * K + p
    x = seeded((B, C, L), 1000 + sd, tdt); w = seeded((C, K), 2000 + sd, tdt); dy = seeded((B, C, L), 3000 + sd, tdt)
    xd, wd, dyd = x.cuda(), w.cuda(), dy.cuda()
    dx, dw = binding.dwconv_bwd(dyd, xd, wd, p)
    dx_sep = binding.dwconv_bwd_input(dyd, wd, p)
    torch.cuda.synchronize()
    assert torch.equal(dx, dx_sep)
    from _parity import normalised_error
    from paper_2604_25422_amd.workloads import as_f32_numpy
    ref, ra = oracle_mod.bwd_weight(as_f32_numpy(x), as_f32_numpy(dy), K, p)
    e, i = normalised_error(dw.float().cpu().numpy().astype(np.float64), ref, ra)
    assert e <= TOL[(dtype, "dw")], f"fused dw err {e:.3e} at {i}"


@pytest.mark.parametrize("B,C,L,K,p,dtype", [(4, 64, 1024, 16, 15, "f32"), (3, 5, 96, 48, 24, "f32"),
                                              (2, 3, 512, 300, 299, "f32"), (4, 6, 1024, 32, 31, "bf16"),
                                              (6, 8, 256, 256, 255, "f32"), (40, 8, 96, 96, 48, "bf16"),
                                              (3, 2, 1024, 2000, 1000, "f32"), (9, 4, 200, 48, 24, "bf16")])
def test_calls_can_be_captured_in_a_graph(B, C, L, K, p, dtype):
    """Every entry point only enqueues kernels (no allocation, no synchronisation, no memset nodes), so a step can
    be captured once and replayed; replays, with eager work in between, give the bits of the eager calls."""
    from paper_2604_25422_amd import binding
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = seeded((B, C, L), 41, tdt).cuda(); w = seeded((C, K), 42, tdt).cuda(); dy = seeded((B, C, L), 43, tdt).cuda()
    y = torch.empty_like(x); dx = torch.empty_like(x); dw = torch.empty_like(w)
    dx2 = torch.empty_like(x); dw2 = torch.empty_like(w)
    ws = binding.new_workspace(x, K, p)

    def step():
        binding.dwconv_fwd(x, w, p, out=y)
        binding.dwconv_bwd_input(dy, w, p, out=dx)
        binding.dwconv_bwd_weight(x, dy, K, p, workspace=ws, out=dw)
        binding.dwconv_bwd(dy, x, w, p, workspace=ws, out_dx=dx2, out_dw=dw2)

    step()                      # eager: also warms the per-kernel caches of the library
    torch.cuda.synchronize()
    ref = [t.clone() for t in (y, dx, dw, dx2, dw2)]
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(g, stream=side):
        step()
    for rep in range(3):
        for t in (y, dx, dw, dx2, dw2):
            t.fill_(float("nan"))           # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for name, t, r in zip(("y", "dx", "dw", "dx fused", "dw fused"), (y, dx, dw, dx2, dw2), ref):
            assert torch.equal(t, r), f"replay {rep}: {name} differs from the eager call"


def test_binding_rejects_mismatched_outputs():
    """The marshalling layer checks what the C ABI cannot see: shapes and types of caller-supplied outputs."""
    from paper_2604_25422_amd import binding
    B, C, L, K, p = 2, 3, 64, 9, 4
    x = torch.zeros((B, C, L), device="cuda"); w = torch.zeros((C, K), device="cuda")
    with pytest.raises(ValueError):
        binding.dwconv_bwd_weight(x, x, K, p, out=torch.zeros((C, K - 1), device="cuda"))
    with pytest.raises(TypeError):
        binding.dwconv_bwd_weight(x, x, K, p, out=torch.zeros((C, K), device="cuda", dtype=torch.bfloat16))
    with pytest.raises(TypeError):
        binding.dwconv_bwd(x, x, w.to(torch.bfloat16), p)
    with pytest.raises(ValueError):
        binding.dwconv_bwd(x, x, w, p, out_dw=torch.zeros((C, K + 1), device="cuda"))
    with pytest.raises(ValueError):
        binding.dwconv_bwd_weight_finalize(torch.zeros(1024, dtype=torch.uint8), B, C, L, K, p, torch.float32)   # host workspace
    with pytest.raises(ValueError):
        binding.dwconv_fwd(x.cpu(), w, p)


def test_first_calls_of_a_process_can_be_captured():
    """Capture WITHOUT a preceding eager call: the library's per-kernel occupancy and LDS-attribute queries then run
    while the stream is capturing.  A fresh process, so that no kernel has been launched before."""
    import subprocess
    import sys
    code = r"""
import sys, torch
sys.path.insert(0, %r); sys.path.insert(0, %r)
from _parity import seeded
from paper_2604_25422_amd import binding
for (B, C, L, K, p, dt) in ((4, 64, 1024, 16, 15, torch.float32), (3, 5, 96, 48, 24, torch.float32),
                            (2, 3, 512, 300, 299, torch.float32), (4, 6, 1024, 32, 31, torch.bfloat16),
                            (2, 2, 2048, 100, 99, torch.float32)):
    x = seeded((B, C, L), 41, dt).cuda(); w = seeded((C, K), 42, dt).cuda(); dy = seeded((B, C, L), 43, dt).cuda()
    y = torch.empty_like(x); dx = torch.empty_like(x); dw = torch.empty_like(w); dx2 = torch.empty_like(x); dw2 = torch.empty_like(w)
    ws = binding.new_workspace(x, K, p)
    def step():
        binding.dwconv_fwd(x, w, p, out=y)
        binding.dwconv_bwd_input(dy, w, p, out=dx)
        binding.dwconv_bwd_weight(x, dy, K, p, workspace=ws, out=dw)
        binding.dwconv_bwd(dy, x, w, p, workspace=ws, out_dx=dx2, out_dw=dw2)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        step()
    outs = (y, dx, dw, dx2, dw2)
    got = []
    for rep in range(2):
        for t in outs: t.fill_(float("nan"))
        torch.cuda.synchronize(); g.replay(); torch.cuda.synchronize()
        got.append([t.clone() for t in outs])
    step(); torch.cuda.synchronize()
    for rep in range(2):
        for a, b in zip(got[rep], outs):
            assert torch.equal(a, b), (B, C, L, K, rep)
print("CAPTURE_OK")
""" % (os.path.dirname(os.path.dirname(os.path.abspath(__file__))), os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=240)
    assert r.returncode == 0 and "CAPTURE_OK" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]
