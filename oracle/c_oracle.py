"""ctypes loader for the plain C oracle (oracle/mq_oracle.c).

TEST INFRASTRUCTURE ONLY.  build() compiles it with gcc; the product never
loads it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mq_oracle.c")
_LIB = os.path.join(_HERE, "libmq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.mqo_slice.restype = ctypes.c_int
        lib.mqo_slice.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                  ctypes.c_void_p]
        lib.mqo_linear.restype = ctypes.c_int
        lib.mqo_linear.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                   ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        _lib = lib
    return _lib


def slice_codes(q, c: int, r: int) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.uint8)
    S = np.empty_like(q)
    rc = _load().mqo_slice(q.ctypes.data, q.size, c, r, S.ctypes.data)
    if rc != 0:
        raise ValueError("mqo_slice rejected its arguments")
    return S


def linear(x, parent, scales, zeros, c: int, r: int, group: int):
    """Returns (y float64 [M,N], threads_used)."""
    x = np.ascontiguousarray(x, dtype=np.float16)
    parent = np.ascontiguousarray(parent, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float16)
    zeros = np.ascontiguousarray(zeros, dtype=np.float16)
    M, K = x.shape
    N = parent.shape[0]
    y = np.empty((M, N), dtype=np.float64)
    used = _load().mqo_linear(x.ctypes.data, M, parent.ctypes.data, scales.ctypes.data,
                              zeros.ctypes.data, N, K, c, r, group, y.ctypes.data)
    if used < 0:
        raise ValueError("mqo_linear rejected its arguments")
    return y, used
