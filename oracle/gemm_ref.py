"""Loader for the C triple-loop reference GEMM (oracle/gemm_ref.c).

TEST INFRASTRUCTURE ONLY: used by tests, the smoke check and the benchmark's
cpu_baseline leg for shapes where numpy's int64 matmul is too slow.  Built with
gcc; shares nothing with the HIP library."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_ref.c")
_LIB = os.path.join(_HERE, "liboracle_gemm.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        i64 = ctypes.c_int64
        _lib.oracle_gemm_i8_i64.argtypes = [ctypes.c_void_p, ctypes.c_void_p, i64, i64, i64, ctypes.c_void_p]
        _lib.oracle_gemm_i8_i64.restype = None
        _lib.oracle_gemm_f64.argtypes = [ctypes.c_void_p, ctypes.c_void_p, i64, i64, i64, ctypes.c_void_p]
        _lib.oracle_gemm_f64.restype = None
        _lib.oracle_omp_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_load().oracle_omp_threads())


def gemm_i8_i64(Xq: np.ndarray, Wq: np.ndarray) -> np.ndarray:
    """acc[m, o] = sum_k Xq[m, k] * Wq[o, k] in int64 (int8 operands)."""
    X = np.ascontiguousarray(Xq, dtype=np.int8)
    W = np.ascontiguousarray(Wq, dtype=np.int8)
    M, K = X.shape
    O, K2 = W.shape
    assert K == K2
    acc = np.empty((M, O), dtype=np.int64)
    _load().oracle_gemm_i8_i64(X.ctypes.data, W.ctypes.data, M, O, K, acc.ctypes.data)
    return acc


def gemm_f64(Xd: np.ndarray, Wd: np.ndarray) -> np.ndarray:
    """acc[m, o] = sum_k Xd[m, k] * Wd[o, k] in fp64, k ascending."""
    X = np.ascontiguousarray(Xd, dtype=np.float64)
    W = np.ascontiguousarray(Wd, dtype=np.float64)
    M, K = X.shape
    O, K2 = W.shape
    assert K == K2
    acc = np.empty((M, O), dtype=np.float64)
    _load().oracle_gemm_f64(X.ctypes.data, W.ctypes.data, M, O, K, acc.ctypes.data)
    return acc
