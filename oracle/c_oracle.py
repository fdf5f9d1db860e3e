"""ctypes loader for the plain-C fp64 oracle (oracle/hlq_oracle.c).  TEST INFRASTRUCTURE ONLY.

`build()` compiles the C file with gcc; `gemm_f64` calls it.  Used where the numpy
oracle would need too much memory or time (full-size shapes, the CPU baseline)."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hlq_oracle.c")
_LIB = os.path.join(_HERE, "libhlq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.hlq_oracle_gemm_f64.restype = ctypes.c_int
        lib.hlq_oracle_gemm_f64.argtypes = [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64]
        lib.hlq_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().hlq_oracle_num_threads())


def gemm_f64(X, codes, scales, zeros, q: int, G: int, cols=None) -> np.ndarray:
    """Y[M, ncols] fp64 = X @ W^ restricted to `cols` (all columns if None)."""
    lib = _load()
    X = np.ascontiguousarray(X, dtype=np.float16)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float16)
    zeros = np.ascontiguousarray(zeros, dtype=np.float16)
    M, K = X.shape
    N = codes.shape[1]
    assert codes.shape == (K, N) and scales.shape == (q, K // G, N) and zeros.shape == (K // G, N)
    if cols is not None:
        cols = np.ascontiguousarray(cols, dtype=np.int64)
        ncols = cols.shape[0]
        cptr = cols.ctypes.data
    else:
        ncols, cptr = N, None
    Y = np.empty((M, ncols), dtype=np.float64)
    rc = lib.hlq_oracle_gemm_f64(K, N, q, G, M, codes.ctypes.data, scales.ctypes.data,
                                 zeros.ctypes.data, X.ctypes.data, K,
                                 Y.ctypes.data, ncols, cptr, ncols)
    if rc != 0:
        raise ValueError("hlq_oracle_gemm_f64: bad argument")
    return Y
