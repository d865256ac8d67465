"""ctypes front end of oracle/conv_oracle.c (TEST INFRASTRUCTURE ONLY).

`build()` compiles the C file with gcc into oracle/libconv_oracle.so; `load()` opens it
(building first if it is missing).  The wrappers take integer numpy arrays of fixed-point
codes (NHWC / KRSC) and return int64 arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "libconv_oracle.so")
_lib = None


class _Shape(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int) for f in ("n", "h", "w", "c", "k", "r", "s", "stride", "pad")]


def build() -> str:
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall",
                           "-o", _LIB, _SRC])
    return _LIB


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
            build()
        _lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        _lib.oracle_gemm.argtypes = [ctypes.c_int] * 3 + [i32p, i32p, i64p]
        for f in (_lib.oracle_conv_fwd, _lib.oracle_conv_dgrad, _lib.oracle_conv_wgrad):
            f.argtypes = [_Shape, i32p, i32p, i64p]
            f.restype = None
        _lib.oracle_gemm.restype = None
    return _lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _out(shape):
    o = np.empty(shape, dtype=np.int64)
    return o, o.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _dims(n, h, w, c, k, r, s, stride, pad):
    return (h + 2 * pad - r) // stride + 1, (w + 2 * pad - s) // stride + 1


def gemm(a, b) -> np.ndarray:
    a, pa = _i32(a)
    b, pb = _i32(b)
    m, k = a.shape
    k2, n = b.shape
    assert k == k2
    c, pc = _out((m, n))
    load().oracle_gemm(m, n, k, pa, pb, pc)
    return c


def conv_fwd(x, w, stride: int = 1, pad: int = 1) -> np.ndarray:
    x, px = _i32(x)
    w, pw = _i32(w)
    n, h, wd, c = x.shape
    k, r, s, c2 = w.shape
    assert c == c2
    p, q = _dims(n, h, wd, c, k, r, s, stride, pad)
    y, py = _out((n, p, q, k))
    load().oracle_conv_fwd(_Shape(n, h, wd, c, k, r, s, stride, pad), px, pw, py)
    return y


def conv_dgrad(dy, w, h: int, wd: int, stride: int = 1, pad: int = 1) -> np.ndarray:
    dy, pdy = _i32(dy)
    w, pw = _i32(w)
    n, p, q, k = dy.shape
    k2, r, s, c = w.shape
    assert k == k2 and (p, q) == _dims(n, h, wd, c, k, r, s, stride, pad)
    dx, pdx = _out((n, h, wd, c))
    load().oracle_conv_dgrad(_Shape(n, h, wd, c, k, r, s, stride, pad), pdy, pw, pdx)
    return dx


def conv_wgrad(dy, x, r: int, s: int, stride: int = 1, pad: int = 1) -> np.ndarray:
    dy, pdy = _i32(dy)
    x, px = _i32(x)
    n, p, q, k = dy.shape
    n2, h, wd, c = x.shape
    assert n == n2 and (p, q) == _dims(n, h, wd, c, k, r, s, stride, pad)
    dw, pdw = _out((k, r, s, c))
    load().oracle_conv_wgrad(_Shape(n, h, wd, c, k, r, s, stride, pad), pdy, px, pdw)
    return dw


def num_threads() -> int:
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
