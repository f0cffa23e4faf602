"""CPU-only checks of the C ABI: the shared library loads, exports every symbol the header
declares, and validates its arguments before touching HIP (so error paths run without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2604_25422_amd import _build, binding
    if _build.is_stale():
        _build.build()
    return binding.lib()


def header_symbols():
    text = open(os.path.join(ROOT, "include", "dwconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dwconv_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2604_25422_amd import binding
    syms = header_symbols()
    assert len(syms) >= 9
    assert set(syms) == set(binding.SYMBOLS)
    for s in syms:
        assert hasattr(lib, s), s


def test_version_and_status_strings(lib):
    assert lib.dwconv_version() >= 100
    seen = set()
    for code in range(0, 9):
        s = lib.dwconv_status_string(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert lib.dwconv_status_string(99).decode() == "unknown status"


P = 0x1000  # any non-NULL, aligned, never-dereferenced address: validation fails before a launch


@pytest.mark.parametrize("fn", ["dwconv_fwd", "dwconv_bwd_input"])
def test_corr_argument_validation(lib, fn):
    f = getattr(lib, fn)
    assert f(None, P, P, 1, 1, 8, 3, 1, 0, None) == 1
    assert f(P, None, P, 1, 1, 8, 3, 1, 0, None) == 1
    assert f(P, P, None, 1, 1, 8, 3, 1, 0, None) == 1
    assert f(P, P, P, 0, 1, 8, 3, 1, 0, None) == 2
    assert f(P, P, P, 1, 0, 8, 3, 1, 0, None) == 2
    assert f(P, P, P, 1, 1, 0, 3, 1, 0, None) == 2
    assert f(P, P, P, 1, 1, 8, 0, 0, 0, None) == 2
    assert f(P, P, P, 1 << 20, 1 << 20, 8, 3, 1, 0, None) == 2
    assert f(P, P, P, 1, 1, 8, 3, 3, 0, None) == 3
    assert f(P, P, P, 1, 1, 8, 3, -1, 0, None) == 3
    assert f(P, P, P, 1, 1, 8, 3, 1, 2, None) == 4
    assert f(P + 2, P, P, 1, 1, 8, 3, 1, 0, None) == 6
    assert f(P, P, P + 1, 1, 1, 8, 3, 1, 1, None) == 6


def test_weight_gradient_argument_validation(lib):
    need = lib.dwconv_bwd_weight_workspace_bytes(2, 3, 100, 5, 2, 0)
    assert need >= lib.dwconv_bwd_weight_slices(2, 3, 100, 5, 2, 0) * 3 * 5 * 4 > 0
    f = lib.dwconv_bwd_weight
    assert f(None, P, P, P, need, 2, 3, 100, 5, 2, 0, None) == 1
    assert f(P, P, None, P, need, 2, 3, 100, 5, 2, 0, None) == 1
    assert f(P, P, P, P, need, 2, 3, 100, 0, 0, 0, None) == 2
    assert f(P, P, P, P, need, 2, 3, 100, 5, 5, 0, None) == 3
    assert f(P, P, P, P, need, 2, 3, 100, 5, 2, 7, None) == 4
    assert f(P, P, P, None, need, 2, 3, 100, 5, 2, 0, None) == 5
    assert f(P, P, P, P, need - 1, 2, 3, 100, 5, 2, 0, None) == 5
    assert f(P, P, P, P + 4, need, 2, 3, 100, 5, 2, 0, None) == 5
    assert f(P + 1, P, P, P, need, 2, 3, 100, 5, 2, 0, None) == 6
    assert lib.dwconv_bwd_weight_partial(P, P, P, need - 1, 2, 3, 100, 5, 2, 0, None) == 5
    assert lib.dwconv_bwd_weight_finalize(P, need - 1, P, 2, 3, 100, 5, 2, 0, None) == 5
    assert lib.dwconv_bwd_weight_finalize(P, need, None, 2, 3, 100, 5, 2, 0, None) == 1


def test_fused_backward_argument_validation(lib):
    need = lib.dwconv_bwd_weight_workspace_bytes(2, 3, 100, 5, 2, 0)
    f = lib.dwconv_bwd          # (dy, x, w, dx, dw, workspace, bytes, B, C, L, K, pad, dtype, stream)
    for missing in range(5):
        args = [P] * 5
        args[missing] = None
        assert f(*args, P, need, 2, 3, 100, 5, 2, 0, None) == 1
    assert f(P, P, P, P, P, P, need, 0, 3, 100, 5, 2, 0, None) == 2
    assert f(P, P, P, P, P, P, need, 2, 3, 100, 5, 5, 0, None) == 3
    assert f(P, P, P, P, P, P, need, 2, 3, 100, 5, 2, 9, None) == 4
    assert f(P, P, P, P, P, None, need, 2, 3, 100, 5, 2, 0, None) == 5
    assert f(P, P, P, P, P, P, need - 1, 2, 3, 100, 5, 2, 0, None) == 5
    assert f(P, P, P, P + 2, P, P, need, 2, 3, 100, 5, 2, 0, None) == 6
    # which shapes take the fused kernel: filters of the register-resident class, row length a multiple of 4 (fp32)
    q = lib.dwconv_bwd_is_fused
    assert q(32, 256, 4096, 64, 63, 0) == 1 and q(4096, 128, 196, 48, 24, 0) == 1 and q(2, 3, 200, 5, 2, 0) == 1
    assert q(128, 768, 1024, 32, 31, 1) == 1 and q(2, 3, 100, 5, 2, 1) == 1     # bf16: rows of whole 8-byte granules
    assert q(2, 3, 102, 5, 2, 1) == 1 and q(2, 3, 101, 5, 2, 1) == 0 and q(2, 3, 60, 5, 2, 1) == 0
    assert q(8, 256, 8192, 8192, 8191, 0) == 0 and q(2, 3, 101, 5, 2, 0) == 0
    assert q(2, 3, 100, 2, 1, 0) == 0 and q(0, 3, 100, 5, 2, 0) == 0
    assert q(16384, 128, 48, 48, 24, 0) == 1        # rows of at most 64 positions: sixteen rows per tile
    # bf16 virtual rows: rows of even length
    assert q(4096, 128, 200, 48, 24, 1) == 1 and q(4096, 128, 196, 48, 24, 1) == 1 and q(4096, 128, 198, 48, 24, 1) == 1
    assert q(4096, 128, 199, 48, 24, 1) == 0


def test_workspace_query_rejects_bad_shapes(lib):
    assert lib.dwconv_bwd_weight_workspace_bytes(0, 3, 100, 5, 2, 0) == 0
    assert lib.dwconv_bwd_weight_workspace_bytes(2, 3, 100, 5, 9, 0) == 0
    assert lib.dwconv_bwd_weight_slices(2, 3, 100, 5, 2, 3) == 0
    for (B, C, L, K, p, dt) in [(32, 256, 4096, 64, 63, 0), (64, 512, 2048, 7, 3, 0), (8, 256, 8192, 8192, 8191, 0),
                                (128, 768, 1024, 32, 31, 1), (1, 1, 1, 1, 0, 0), (16384, 128, 48, 48, 24, 0),
                                (3, 5, 600, 64, 63, 0), (32, 256, 4096, 256, 255, 0), (32, 256, 4096, 600, 0, 0),
                                (32, 256, 4096, 994, 993, 1), (128, 768, 1024, 512, 511, 1), (2, 4, 1024, 300, 150, 1),
                                (64, 256, 512, 300, 150, 1), (5, 3, 4100, 700, 350, 1)]:
        S = lib.dwconv_bwd_weight_slices(B, C, L, K, p, dt)
        n = lib.dwconv_bwd_weight_workspace_bytes(B, C, L, K, p, dt)
        assert S >= 1 and n >= S * C * K * 4 and n % 16 == 0
    # rows of at most 48 positions: the fused backward call writes one slice per wave (about 4096 / C per channel),
    # more than the separate weight-gradient call; the query covers both
    assert lib.dwconv_bwd_weight_workspace_bytes(16384, 128, 48, 48, 24, 0) >= 32 * 128 * 48 * 4
    assert lib.dwconv_bwd_weight_workspace_bytes(16384, 128, 48, 48, 24, 1) >= 32 * 128 * 48 * 4
    assert lib.dwconv_bwd_is_fused(16384, 128, 48, 48, 24, 1) == 1 and lib.dwconv_bwd_is_fused(4096, 8, 60, 16, 8, 1) == 0


def test_single_pass_query(lib):
    # whole-channel workgroups: C a small multiple of the 256 compute units, enough segments per wave
    f = lib.dwconv_bwd_weight_single_pass
    assert f(32, 256, 4096, 64, 63, 0) == 1 and lib.dwconv_bwd_weight_slices(32, 256, 4096, 64, 63, 0) == 1
    assert f(64, 512, 2048, 7, 3, 0) == 1
    assert f(128, 768, 1024, 32, 31, 1) == 1
    assert f(40, 64, 1024, 16, 15, 0) == 0           # channels do not fill the chip
    assert f(4, 64, 1024, 16, 15, 0) == 1            # ... but at most four segments per wave: launch-bound, one kernel
    assert f(8, 256, 8192, 8192, 8191, 0) == 0       # long filter: two zero-filled slices
    assert f(1, 256, 1024, 16, 15, 0) == 1           # a single segment per channel: one kernel as well
    assert f(32, 256, 4098, 64, 63, 0) == 1          # row length not a multiple of 4: rows still start on a dword
    assert f(32, 256, 4098, 128, 127, 0) == 0        # ... but only up to six block offsets
    assert f(128, 768, 1026, 32, 31, 1) == 1 and f(128, 768, 1025, 32, 31, 1) == 0      # bf16: even lengths
    assert lib.dwconv_bwd_is_fused(32, 256, 4098, 64, 63, 0) == 1 and lib.dwconv_bwd_is_fused(32, 256, 4097, 64, 63, 1) == 0
    # short rows that are not whole granules: virtual rows (fp32 any length, bf16 even lengths), fused
    assert lib.dwconv_bwd_is_fused(4, 8, 500, 64, 63, 0) == 1 and lib.dwconv_bwd_is_fused(4, 8, 502, 64, 63, 0) == 1
    assert lib.dwconv_bwd_is_fused(4, 8, 503, 64, 63, 0) == 1 and lib.dwconv_bwd_is_fused(4, 8, 503, 64, 63, 1) == 0
    assert lib.dwconv_bwd_is_fused(4, 8, 502, 128, 127, 0) == 0      # ... up to six block offsets
    # seventeen to thirty-two block offsets: two launches over halves of the offsets, each into its own slices,
    # so an even number of slices and never one kernel - also for small problems, in either storage type
    S226, S256 = lib.dwconv_bwd_weight_slices(32, 256, 4096, 226, 225, 0), lib.dwconv_bwd_weight_slices(32, 256, 4096, 256, 255, 0)
    assert S256 == 2 * S226 and f(32, 256, 4096, 256, 255, 0) == 0
    assert f(2, 4, 1024, 300, 150, 0) == 0 and lib.dwconv_bwd_weight_slices(2, 4, 1024, 300, 150, 0) == 2
    assert lib.dwconv_bwd_weight_slices(32, 256, 4096, 256, 255, 1) == S256
    # bf16: up to four launches (up to 64 offsets), fp32 up to three (48); beyond, the long-filter kernel: two slices per
    # batch slice (one batch slice where channels x offset groups already fill the chip, as on the benchmark shape)
    assert lib.dwconv_bwd_weight_slices(32, 256, 4096, 994, 993, 1) == 2 * S256
    assert lib.dwconv_bwd_weight_slices(32, 256, 4096, 994, 993, 0) == 4
    assert lib.dwconv_bwd_weight_slices(8, 256, 8192, 8192, 8191, 0) == 2
    assert lib.dwconv_bwd_weight_slices(1000, 1, 1024, 2000, 1000, 0) == 250    # one channel: 125 batch slices of eight rows
    assert 2 * lib.dwconv_bwd_weight_slices(32, 256, 4096, 600, 599, 0) == 3 * S256
    # ... but not for rows that fill less than three quarters of their segments (long-filter kernel: two slices per batch slice)
    assert lib.dwconv_bwd_weight_slices(64, 256, 640, 300, 150, 0) == 4 and f(64, 256, 640, 300, 150, 0) == 0
    assert f(0, 256, 4096, 64, 63, 0) == 0           # bad shape


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_2604_25422_amd import binding
    x = torch.zeros(1, 2, 8); w = torch.zeros(2, 3)
    with pytest.raises(ValueError):
        binding.dwconv_fwd(x, w, 1)
    with pytest.raises(ValueError):
        binding.dwconv_bwd_input(x, w, 1)
    with pytest.raises(ValueError):
        binding.dwconv_bwd_weight(x, x, 3, 1)


def test_workloads_are_seeded_and_shaped():
    import torch
    from paper_2604_25422_amd import workloads
    assert len(workloads.WORKLOADS) == 9 and workloads.HEADLINE.K == 64
    wl = workloads.WORKLOADS[0]
    a = workloads.make_inputs(wl); b = workloads.make_inputs(wl)
    for k in ("x", "w", "dy"):
        assert torch.equal(a[k], b[k])
    assert a["x"].shape == (4, 64, 1024) and a["w"].shape == (64, 16) and a["x"].dtype == torch.float32
    assert not torch.equal(a["x"], a["dy"])
    w3 = workloads.make_filter(workloads.WORKLOADS[3].with_shape(C=4))
    assert w3.shape == (4, 8192) and float(w3[:, 0].min()) == 1.0 and float(w3.abs().max()) <= 1.0
    w4 = workloads.make_filter(workloads.WORKLOADS[4])
    assert w4.dtype == torch.bfloat16


def test_noalloc_argument_validation(lib):
    """The allocation-free weight gradient validates like dwconv_bwd_weight and turns away shapes whose partial
    sums do not fit the built-in scratch, all before any HIP call."""
    f = lib.dwconv_bwd_weight_noalloc
    cap = lib.dwconv_noalloc_scratch_bytes()
    assert cap == 16 << 20
    assert f(None, P, P, 2, 3, 100, 5, 2, 0, None) == 1
    assert f(P, P, None, 2, 3, 100, 5, 2, 0, None) == 1
    assert f(P, P, P, 2, 3, 100, 0, 0, 0, None) == 2
    assert f(P, P, P, 2, 3, 100, 5, 5, 0, None) == 3
    assert f(P, P, P, 2, 3, 100, 5, 2, 7, None) == 4
    assert f(P + 1, P, P, 2, 3, 100, 5, 2, 0, None) == 6
    assert lib.dwconv_bwd_weight_workspace_bytes(1, 512, 8192, 8192, 8191, 0) > cap
    assert f(P, P, P, 1, 512, 8192, 8192, 8191, 0, None) == 8
    # every benchmark shape fits
    for shape in ((4, 64, 1024, 16, 15, 0), (32, 256, 4096, 64, 63, 0), (64, 512, 2048, 7, 3, 0),
                  (8, 256, 8192, 8192, 8191, 0), (128, 768, 1024, 32, 31, 1), (16384, 128, 48, 48, 24, 0)):
        assert 0 < lib.dwconv_bwd_weight_workspace_bytes(*shape) <= cap, shape
