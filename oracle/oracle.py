"""Loader for the C oracle (gemm_oracle.c).  TEST INFRASTRUCTURE ONLY.

C[i][j] = sum_t A[i][t] * B[t][j] over unpacked int8 with int32 accumulation --
the definition of the product that the paper's Section II-A names C = AB and that
its binary/ternary algorithms (Section III, eq. (6) and (7)) compute exactly.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile gemm_oracle.c with gcc (-O3, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC])
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_gemm_i8_i32.argtypes = [i64, i64, i64, p, p, p, ctypes.c_int]
        lib.oracle_gemm_i8_i32.restype = ctypes.c_int
        lib.oracle_gemm_i8_i32_samples.argtypes = [i64, i64, p, p, i64, p, p, p]
        lib.oracle_gemm_i8_i32_samples.restype = None
        lib.oracle_gemm_u8_zp_i32.argtypes = [i64, i64, i64, p, p, ctypes.c_int32, ctypes.c_int32, p]
        lib.oracle_gemm_u8_zp_i32.restype = None
        _lib = lib
    return _lib


def _check(A: np.ndarray, B: np.ndarray) -> Tuple[int, int, int]:
    if A.dtype != np.int8 or B.dtype != np.int8:
        raise TypeError("oracle takes int8 matrices")
    if A.ndim != 2 or B.ndim != 2 or A.shape[1] != B.shape[0]:
        raise ValueError("shape mismatch")
    if not (A.flags.c_contiguous and B.flags.c_contiguous):
        raise ValueError("oracle takes C-contiguous matrices")
    return A.shape[0], B.shape[1], A.shape[1]


def gemm(A: np.ndarray, B: np.ndarray, threads: int = 0) -> np.ndarray:
    """Full product, int32 M x N."""
    M, N, K = _check(A, B)
    C = np.empty((M, N), dtype=np.int32)
    if M and N:
        _load().oracle_gemm_i8_i32(M, N, K, A.ctypes.data, B.ctypes.data, C.ctypes.data, int(threads))
    return C


def gemm_threads(A: np.ndarray, B: np.ndarray, threads: int = 0) -> Tuple[np.ndarray, int]:
    """Like gemm() but also returns the number of threads OpenMP used."""
    M, N, K = _check(A, B)
    C = np.empty((M, N), dtype=np.int32)
    used = _load().oracle_gemm_i8_i32(M, N, K, A.ctypes.data, B.ctypes.data, C.ctypes.data, int(threads))
    return C, int(used)


def gemm_samples(A: np.ndarray, B: np.ndarray, ii: np.ndarray, jj: np.ndarray) -> np.ndarray:
    """out[s] = (A B)[ii[s], jj[s]] for selected entries."""
    M, N, K = _check(A, B)
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    if ii.shape != jj.shape or ii.ndim != 1:
        raise ValueError("ii, jj must be equal-length vectors")
    if len(ii) and (ii.min() < 0 or ii.max() >= M or jj.min() < 0 or jj.max() >= N):
        raise IndexError("sample index out of range")
    out = np.empty(len(ii), dtype=np.int32)
    _load().oracle_gemm_i8_i32_samples(N, K, A.ctypes.data, B.ctypes.data, len(ii), ii.ctypes.data, jj.ctypes.data,
                                       out.ctypes.data)
    return out


def gemm_u8_zero_point(A: np.ndarray, B: np.ndarray, zA: int, zB: int) -> np.ndarray:
    """C[i][j] = sum_t (A[i][t] - zA)(B[t][j] - zB) for uint8 matrices (eq. (2)/(3) of the paper, left-hand side)."""
    if A.dtype != np.uint8 or B.dtype != np.uint8:
        raise TypeError("uint8 matrices expected")
    if A.ndim != 2 or B.ndim != 2 or A.shape[1] != B.shape[0] or not (A.flags.c_contiguous and B.flags.c_contiguous):
        raise ValueError("shape / layout mismatch")
    M, K = A.shape
    N = B.shape[1]
    C = np.empty((M, N), dtype=np.int32)
    if M and N:
        _load().oracle_gemm_u8_zp_i32(M, N, K, A.ctypes.data, B.ctypes.data, int(zA), int(zB), C.ctypes.data)
    return C
