"""CPU fp64 oracle (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It is independent of the HIP path: no shared code, and neither
imports the other.

    build()                       compile codegemm_oracle.c with gcc (+OpenMP)
    gemm(x, codes, codebooks, scales)        -> (y, T)  float64 [B][N]
    dequantize(codes, codebooks, scales)     -> W       float64 [N][K]
scales is [N] (one scale per output row, g = -1) or [N][K/g] (one per run of g weights).
    psumbook(x, codebooks)                   -> P       float64 [B][m][K/v][256]
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "codegemm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the C oracle.  x86-64-v3 rather than -march=native: the library
    is built in one container and may run on another host."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i, p = ctypes.c_int, ctypes.c_void_p
        lib.oracle_num_threads.restype = i
        lib.oracle_set_num_threads.argtypes = [i]
        lib.oracle_set_num_threads.restype = None
        lib.oracle_dequantize.argtypes = [i, i, i, i, i, p, p, p, p]
        lib.oracle_dequantize.restype = i
        lib.oracle_gemm.argtypes = [i, i, i, i, i, i, p, p, p, p, p, p]
        lib.oracle_gemm.restype = i
        lib.oracle_psumbook.argtypes = [i, i, i, i, p, p, p]
        lib.oracle_psumbook.restype = i
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the following calls use (for timing the oracle on one core)."""
    _load().oracle_set_num_threads(int(n))


def _c(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _shapes(codes: np.ndarray, codebooks: np.ndarray) -> Tuple[int, int, int, int]:
    m, N, J = codes.shape
    m2, nc, v = codebooks.shape
    if m2 != m or nc != 256:
        raise ValueError("codebooks must be [m][256][v] with the same m as codes")
    return m, N, J, v


def _group_size(scales: np.ndarray, N: int, K: int) -> int:
    """-1 for scales of shape [N]; K / G for shape [N][G]."""
    if scales.shape == (N,):
        return -1
    if scales.ndim == 2 and scales.shape[0] == N and scales.shape[1] >= 1 and K % scales.shape[1] == 0:
        return K // scales.shape[1]
    raise ValueError("scales must be [N] or [N][K/g]")


def gemm(x: np.ndarray, codes: np.ndarray, codebooks: np.ndarray, scales: np.ndarray):
    """y[b][n] and T[b][n] (sum of |x*W| terms), both float64."""
    x = _c(x, np.float16); codes = _c(codes, np.uint8)
    codebooks = _c(codebooks, np.float16); scales = _c(scales, np.float16)
    m, N, J, v = _shapes(codes, codebooks)
    B, K = x.shape
    if K != J * v:
        raise ValueError("shape mismatch")
    g = _group_size(scales, N, K)
    y = np.empty((B, N), np.float64)
    T = np.empty((B, N), np.float64)
    rc = _load().oracle_gemm(B, N, K, v, m, g, _ptr(x.view(np.uint16)), _ptr(codes),
                             _ptr(codebooks.view(np.uint16)), _ptr(scales.view(np.uint16)), _ptr(y), _ptr(T))
    if rc:
        raise RuntimeError(f"oracle_gemm failed: {rc}")
    return y, T


def dequantize(codes: np.ndarray, codebooks: np.ndarray, scales: np.ndarray) -> np.ndarray:
    codes = _c(codes, np.uint8); codebooks = _c(codebooks, np.float16); scales = _c(scales, np.float16)
    m, N, J, v = _shapes(codes, codebooks)
    W = np.empty((N, J * v), np.float64)
    g = _group_size(scales, N, J * v)
    rc = _load().oracle_dequantize(N, J * v, v, m, g, _ptr(codes), _ptr(codebooks.view(np.uint16)),
                                   _ptr(scales.view(np.uint16)), _ptr(W))
    if rc:
        raise RuntimeError(f"oracle_dequantize failed: {rc}")
    return W


def psumbook(x: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    x = _c(x, np.float16); codebooks = _c(codebooks, np.float16)
    m, nc, v = codebooks.shape
    B, K = x.shape
    if nc != 256 or K % v:
        raise ValueError("shape mismatch")
    P = np.empty((B, m, K // v, 256), np.float64)
    rc = _load().oracle_psumbook(B, K, v, m, _ptr(x.view(np.uint16)), _ptr(codebooks.view(np.uint16)), _ptr(P))
    if rc:
        raise RuntimeError(f"oracle_psumbook failed: {rc}")
    return P
