"""ctypes loader for oracle/direct_conv.c (the float64 direct convolution in C).

Pinned by tests/test_oracle_direct.py against oracle.direct.conv2d_direct and
the brute-force loops.  build() compiles it with gcc -O2 -fopenmp.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle_conv.so")
_lib = None


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "direct_conv.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, src])
    return _SO


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_conv2d_threads.restype = ctypes.c_int
        _lib.oracle_conv2d_f64.restype = None
    return _lib


def threads() -> int:
    return int(_load().oracle_conv2d_threads())


def conv2d_direct_c(x, w, stride=1, pad=0, groups=1, bias=None):
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    assert C == Cg * groups
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    y = np.empty((N, K, P, Q), dtype=np.float64)
    b = None
    if bias is not None:
        b = np.ascontiguousarray(bias, dtype=np.float64)
    fp = ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(ctypes.c_double)
    lib.oracle_conv2d_f64(x.ctypes.data_as(fp), w.ctypes.data_as(fp),
                          b.ctypes.data_as(dp) if b is not None else None,
                          y.ctypes.data_as(dp),
                          *[ctypes.c_int(v) for v in (N, C, H, W, K, R, S, stride, pad, groups)])
    return y
