"""Thin ctypes binding of the C ABI in ``include/dwconv.h`` (argument marshalling only).

Every function takes torch tensors living on the GPU, checks dtype / shape /
contiguity, and hands raw device pointers plus the current HIP stream to the
library.  All arithmetic runs in the HIP kernels; there is no CPU fallback: if
the shared library is missing, loading fails with an error.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import _build

F32 = 0
BF16 = 1

_lib = None

SYMBOLS = (
    "dwconv_fwd", "dwconv_bwd_input", "dwconv_bwd_weight", "dwconv_bwd_weight_partial",
    "dwconv_bwd_weight_finalize", "dwconv_bwd_weight_slices", "dwconv_bwd_weight_single_pass",
    "dwconv_bwd_weight_workspace_bytes", "dwconv_bwd", "dwconv_bwd_is_fused",
    "dwconv_bwd_weight_noalloc", "dwconv_noalloc_scratch_bytes",
    "dwconv_status_string", "dwconv_version",
)


class DwconvError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"dwconv status {status}: {message}")
        self.status = status


def lib():
    """Load ``libdwconv_gfx950.so`` (built in-tree by ``_build.build()``); raise if it is absent."""
    global _lib
    if _lib is None:
        path = _build.LIB_PATH
        if not os.path.exists(path):
            raise FileNotFoundError(
                f"{path} not found: build it first (python -m paper_2604_25422_amd._build, or __graft_entry__.build())")
        l = ctypes.CDLL(path)
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        shape = [i, i, i, i, i, i]
        l.dwconv_fwd.argtypes = [vp, vp, vp] + shape + [vp]
        l.dwconv_bwd_input.argtypes = [vp, vp, vp] + shape + [vp]
        l.dwconv_bwd_weight.argtypes = [vp, vp, vp, vp, sz] + shape + [vp]
        l.dwconv_bwd_weight_partial.argtypes = [vp, vp, vp, sz] + shape + [vp]
        l.dwconv_bwd_weight_finalize.argtypes = [vp, sz, vp] + shape + [vp]
        for n in ("dwconv_fwd", "dwconv_bwd_input", "dwconv_bwd_weight", "dwconv_bwd_weight_partial",
                  "dwconv_bwd_weight_finalize"):
            getattr(l, n).restype = i
        l.dwconv_bwd_weight_slices.argtypes = shape
        l.dwconv_bwd_weight_slices.restype = i
        l.dwconv_bwd.argtypes = [vp, vp, vp, vp, vp, vp, sz] + shape + [vp]
        l.dwconv_bwd.restype = i
        l.dwconv_bwd_is_fused.argtypes = shape
        l.dwconv_bwd_is_fused.restype = i
        l.dwconv_bwd_weight_single_pass.argtypes = shape
        l.dwconv_bwd_weight_single_pass.restype = i
        l.dwconv_bwd_weight_workspace_bytes.argtypes = shape
        l.dwconv_bwd_weight_workspace_bytes.restype = sz
        l.dwconv_bwd_weight_noalloc.argtypes = [vp, vp, vp] + shape + [vp]
        l.dwconv_bwd_weight_noalloc.restype = i
        l.dwconv_noalloc_scratch_bytes.argtypes = []
        l.dwconv_noalloc_scratch_bytes.restype = sz
        l.dwconv_status_string.argtypes = [i]
        l.dwconv_status_string.restype = ctypes.c_char_p
        l.dwconv_version.argtypes = []
        l.dwconv_version.restype = i
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().dwconv_status_string(int(status)).decode()


def _check(status: int):
    if status != 0:
        raise DwconvError(status, status_string(status))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}: float32 or bfloat16 storage only")


def _on_current_device(t: torch.Tensor, name: str):
    """The library enqueues on the current stream of the current device: every tensor must live there."""
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.device.index != torch.cuda.current_device():
        raise ValueError(f"{name} is on {t.device}, the current device is cuda:{torch.cuda.current_device()}")


def _dev3(t: torch.Tensor, name: str):
    _on_current_device(t, name)
    if t.dim() != 3 or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous [B, C, L] tensor")
    return t


def _dev2(t: torch.Tensor, name: str, C: int, K: int | None = None, dtype=None):
    _on_current_device(t, name)
    if t.dim() != 2 or not t.is_contiguous() or t.shape[0] != C:
        raise ValueError(f"{name} must be a contiguous [C, K] tensor")
    if K is not None and t.shape[1] != K:
        raise ValueError(f"{name} must have {K} columns, has {t.shape[1]}")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, is {t.dtype}")
    return t


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def dwconv_fwd(x: torch.Tensor, w: torch.Tensor, pad_left: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """y[b,c,t] = sum_j x~[b,c,t+j-pad_left] w[c,j]  (Sec. IV-A eq. (dwconv))."""
    _dev3(x, "x"); B, C, L = x.shape
    _dev2(w, "w", C); K = w.shape[1]
    if w.dtype != x.dtype:
        raise TypeError("x and w must share a dtype")
    y = torch.empty_like(x) if out is None else _dev3(out, "out")
    if y.shape != x.shape or y.dtype != x.dtype:
        raise ValueError("out must match x")
    _check(lib().dwconv_fwd(x.data_ptr(), w.data_ptr(), y.data_ptr(), B, C, L, K, int(pad_left), _dtype_code(x), _stream()))
    return y


def dwconv_bwd_input(dy: torch.Tensor, w: torch.Tensor, pad_left: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """dx[b,c,s] = sum_j dy~[b,c,s-j+pad_left] w[c,j]  (adjoint of eq. (dwconv); cf. eq. (dx_def))."""
    _dev3(dy, "dy"); B, C, L = dy.shape
    _dev2(w, "w", C); K = w.shape[1]
    if w.dtype != dy.dtype:
        raise TypeError("dy and w must share a dtype")
    dx = torch.empty_like(dy) if out is None else _dev3(out, "out")
    if dx.shape != dy.shape or dx.dtype != dy.dtype:
        raise ValueError("out must match dy")
    _check(lib().dwconv_bwd_input(dy.data_ptr(), w.data_ptr(), dx.data_ptr(), B, C, L, K, int(pad_left), _dtype_code(dy), _stream()))
    return dx


def dwconv_bwd_weight_slices(B, C, L, K, pad_left, dtype_code) -> int:
    return int(lib().dwconv_bwd_weight_slices(B, C, L, K, pad_left, dtype_code))


def dwconv_bwd_weight_single_pass(B, C, L, K, pad_left, dtype_code) -> bool:
    """True when dwconv_bwd_weight runs as one kernel for this shape (no second stage)."""
    return bool(lib().dwconv_bwd_weight_single_pass(B, C, L, K, pad_left, dtype_code))


def dwconv_bwd_weight_workspace_bytes(B, C, L, K, pad_left, dtype_code) -> int:
    return int(lib().dwconv_bwd_weight_workspace_bytes(B, C, L, K, pad_left, dtype_code))


def new_workspace(x: torch.Tensor, K: int, pad_left: int) -> torch.Tensor:
    """Device workspace (uint8 tensor) large enough for the weight gradient of this shape."""
    B, C, L = x.shape
    n = dwconv_bwd_weight_workspace_bytes(B, C, L, K, int(pad_left), _dtype_code(x))
    if n == 0:
        _check(lib().dwconv_bwd_weight_partial(None, None, None, 0, B, C, L, K, int(pad_left), _dtype_code(x), None) or 2)
    return torch.empty(n, dtype=torch.uint8, device=x.device)


def _dw_args(x, dy, K, pad_left, workspace):
    _dev3(x, "x"); _dev3(dy, "dy")
    if dy.shape != x.shape or dy.dtype != x.dtype:
        raise ValueError("x and dy must match")
    if workspace is None:
        workspace = new_workspace(x, K, pad_left)
    _on_current_device(workspace, "workspace")
    if not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    return workspace, workspace.numel() * workspace.element_size()


def dwconv_bwd_weight(x, dy, K: int, pad_left: int, workspace=None, out=None) -> torch.Tensor:
    """dw[c,j] = sum_b sum_t dy[b,c,t] x~[b,c,t+j-pad_left]  (Sec. IV-A eq. (dk_def)); both stages."""
    workspace, nbytes = _dw_args(x, dy, K, pad_left, workspace)
    B, C, L = x.shape
    dw = torch.empty((C, K), dtype=x.dtype, device=x.device) if out is None else _dev2(out, "out", C, int(K), x.dtype)
    _check(lib().dwconv_bwd_weight(x.data_ptr(), dy.data_ptr(), dw.data_ptr(), workspace.data_ptr(), nbytes,
                                   B, C, L, int(K), int(pad_left), _dtype_code(x), _stream()))
    return dw


def dwconv_noalloc_scratch_bytes() -> int:
    return int(lib().dwconv_noalloc_scratch_bytes())


def dwconv_bwd_weight_noalloc(x, dy, K: int, pad_left: int, out: torch.Tensor) -> torch.Tensor:
    """dwconv_bwd_weight without a workspace: partial sums go to the library's built-in scratch; `out` is the
    caller's [C, K] tensor (the call allocates nothing, so it cannot make one)."""
    _dev3(x, "x"); _dev3(dy, "dy")
    if dy.shape != x.shape or dy.dtype != x.dtype:
        raise ValueError("x and dy must match")
    B, C, L = x.shape
    dw = _dev2(out, "out", C, int(K), x.dtype)
    _check(lib().dwconv_bwd_weight_noalloc(x.data_ptr(), dy.data_ptr(), dw.data_ptr(), B, C, L, int(K), int(pad_left),
                                           _dtype_code(x), _stream()))
    return dw


def dwconv_bwd(dy, x, w, pad_left: int, workspace=None, out_dx=None, out_dw=None):
    """Both gradients in one call (fused kernel where it applies): returns (dx, dw)."""
    K = int(w.shape[1])
    workspace, nbytes = _dw_args(x, dy, K, pad_left, workspace)
    B, C, L = x.shape
    wd = _dev2(w, "w", C, K, x.dtype)
    dx = torch.empty_like(dy) if out_dx is None else _dev3(out_dx, "out_dx")
    dw = torch.empty((C, K), dtype=x.dtype, device=x.device) if out_dw is None else _dev2(out_dw, "out_dw", C, K, x.dtype)
    if dx.shape != dy.shape or dx.dtype != dy.dtype:
        raise ValueError("out_dx must be shaped and typed like dy")
    _check(lib().dwconv_bwd(dy.data_ptr(), x.data_ptr(), wd.data_ptr(), dx.data_ptr(), dw.data_ptr(),
                            workspace.data_ptr(), nbytes, B, C, L, K, int(pad_left), _dtype_code(x), _stream()))
    return dx, dw


def dwconv_bwd_is_fused(B, C, L, K, pad_left, dtype_code) -> bool:
    return bool(lib().dwconv_bwd_is_fused(B, C, L, K, pad_left, dtype_code))


def dwconv_bwd_weight_partial(x, dy, K: int, pad_left: int, workspace=None) -> torch.Tensor:
    """Stage 1: fp32 partial sums [S, C, K] left in the returned workspace (Sec. IV-C/D)."""
    workspace, nbytes = _dw_args(x, dy, K, pad_left, workspace)
    B, C, L = x.shape
    _check(lib().dwconv_bwd_weight_partial(x.data_ptr(), dy.data_ptr(), workspace.data_ptr(), nbytes,
                                           B, C, L, int(K), int(pad_left), _dtype_code(x), _stream()))
    return workspace


def dwconv_bwd_weight_finalize(workspace, B, C, L, K: int, pad_left: int, dtype: torch.dtype, out=None) -> torch.Tensor:
    """Stage 2: dw[c,j] = sum_s part[s,c,j] in increasing s (Sec. IV-C/D)."""
    _on_current_device(workspace, "workspace")
    dw = torch.empty((C, K), dtype=dtype, device=workspace.device) if out is None else _dev2(out, "out", C, int(K), dtype)
    code = _dtype_code(dw)
    _check(lib().dwconv_bwd_weight_finalize(workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                            dw.data_ptr(), B, C, L, int(K), int(pad_left), code, _stream()))
    return dw
