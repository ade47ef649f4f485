"""Loader for the C oracle in conv_ref.c (test infrastructure, never used by the product path).

`conv_ref(x, w, stride, pad, dilation)` evaluates the section-2.1 definition of the layer in
fp64 on NHWC / KRSC fp32 arrays and returns the NPQK result as float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_ref.c")
# CONV_REF_LIB: a differently built copy of the same source (the sanitizer leg of the tests loads one)
_LIB = os.environ.get("CONV_REF_LIB") or os.path.join(_HERE, "libconv_ref.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile conv_ref.c with gcc (OpenMP, no fast-math: the fp64 sum keeps its loop order)."""
    if os.environ.get("CONV_REF_LIB"):
        return _LIB                      # built by whoever set the variable
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.conv_ref_f64.restype = ctypes.c_int
        lib.conv_ref_f64.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int] * 10
        lib.conv_ref_out_dim.restype = ctypes.c_int
        lib.conv_ref_out_dim.argtypes = [ctypes.c_int] * 5
        lib.conv_ref_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def out_dim(size: int, filt: int, stride: int, pad: int, dilation: int) -> int:
    return _load().conv_ref_out_dim(size, filt, stride, pad, dilation)


def threads() -> int:
    return _load().conv_ref_threads()


def conv_ref(x: np.ndarray, w: np.ndarray, stride: int = 1, pad: int = 0, dilation: int = 1) -> np.ndarray:
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    if C2 != C:
        raise ValueError("channel mismatch between x and w")
    P = out_dim(H, R, stride, pad, dilation)
    Q = out_dim(W, S, stride, pad, dilation)
    if P < 1 or Q < 1:
        raise ValueError("empty output")
    y = np.empty((N, P, Q, K), dtype=np.float64)
    rc = lib.conv_ref_f64(x.ctypes.data, w.ctypes.data, y.ctypes.data,
                          N, H, W, C, K, R, S, stride, pad, dilation)
    if rc != 0:
        raise ValueError(f"conv_ref_f64 rejected its arguments (rc={rc})")
    return y
