"""TEST INFRASTRUCTURE ONLY: ctypes loader for the plain-C fp64 CPU oracle.

The oracle (``dwconv_oracle.c``) is the operator definition of the paper's
Sec. IV-A (eqs. (dwconv), (dx_def) read as the adjoint, (dk_def)) written as
plain loops with fp64 accumulation.  Only tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; the product path
(``paper_2604_25422_amd``) never does, and this package never imports it.

Functions take C-contiguous float32 numpy arrays (bf16 inputs are widened
exactly by the caller) and return ``(value, abs_sum)`` as float64 arrays, where
``abs_sum`` is the sum of |term| over the same index set as ``value``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dwconv_oracle.c")
_LIB = os.path.join(_HERE, "libdwconv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over independent outputs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
               "-ffp-contract=off", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        lng = ctypes.c_long
        for name in ("dwconv_oracle_fwd", "dwconv_oracle_bwd_input", "dwconv_oracle_bwd_weight"):
            fn = getattr(lib, name)
            fn.argtypes = [fp, fp, dp, dp, lng, lng, lng, lng, lng]
            fn.restype = ctypes.c_int
        lib.dwconv_oracle_threads.argtypes = []
        lib.dwconv_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    """Threads the oracle's parallel loops use."""
    return int(_load().dwconv_oracle_threads())


def _f32(a, shape):
    a = np.asarray(a)
    if a.dtype != np.float32 or not a.flags.c_contiguous:
        raise TypeError("oracle inputs must be C-contiguous float32 arrays")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _check(rc):
    if rc != 0:
        raise ValueError({1: "null pointer", 2: "bad shape", 3: "pad_left outside [0, K-1]"}.get(rc, f"rc={rc}"))


def fwd(x, w, pad_left: int):
    """Forward y[b,c,t] = sum_j x~[b,c,t+j-p] w[c,j]  (Sec. IV-A, eq. (dwconv))."""
    B, C, L = x.shape
    K = w.shape[1]
    x = _f32(x, (B, C, L)); w = _f32(w, (C, K))
    y = np.empty((B, C, L), np.float64); ya = np.empty((B, C, L), np.float64)
    _check(_load().dwconv_oracle_fwd(_ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float),
                                     _ptr(y, ctypes.c_double), _ptr(ya, ctypes.c_double),
                                     B, C, L, K, int(pad_left)))
    return y, ya


def bwd_input(dy, w, pad_left: int):
    """Input gradient dx[b,c,s] = sum_j dy~[b,c,s-j+p] w[c,j]  (adjoint of eq. (dwconv); cf. eq. (dx_def))."""
    B, C, L = dy.shape
    K = w.shape[1]
    dy = _f32(dy, (B, C, L)); w = _f32(w, (C, K))
    dx = np.empty((B, C, L), np.float64); da = np.empty((B, C, L), np.float64)
    _check(_load().dwconv_oracle_bwd_input(_ptr(dy, ctypes.c_float), _ptr(w, ctypes.c_float),
                                           _ptr(dx, ctypes.c_double), _ptr(da, ctypes.c_double),
                                           B, C, L, K, int(pad_left)))
    return dx, da


def bwd_weight(x, dy, K: int, pad_left: int):
    """Weight gradient dw[c,j] = sum_b sum_t dy[b,c,t] x~[b,c,t+j-p]  (Sec. IV-A, eq. (dk_def))."""
    B, C, L = x.shape
    x = _f32(x, (B, C, L)); dy = _f32(dy, (B, C, L))
    dw = np.empty((C, K), np.float64); da = np.empty((C, K), np.float64)
    _check(_load().dwconv_oracle_bwd_weight(_ptr(x, ctypes.c_float), _ptr(dy, ctypes.c_float),
                                            _ptr(dw, ctypes.c_double), _ptr(da, ctypes.c_double),
                                            B, C, L, int(K), int(pad_left)))
    return dw, da
