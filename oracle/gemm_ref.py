"""fp64 reference GEMM over bf16 bit patterns (test infrastructure only).

C[i][j] = sum_k A[i][k] * B[k][j] with A (M x K), B (K x N), C (M x N): the GEMM of the
paper's case study (SwizzlePerf, Appendix "Case Study: GEMM Swizzling").  The compiled
routine lives in gemm_ref.c; `gemm_tiny` is the same definition as three Python loops, for
small cases and for pinning the C routine.

Acceptance rule for a bf16 result computed with fp32 accumulation:
    |C_gpu - C_ref| <= 1e-2 * |C_ref| + 1e-2      (every element)
"""
from __future__ import annotations

import ctypes
import os
import struct
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgemm_ref.so")
_lib = None

RTOL = 1e-2
ATOL = 1e-2


def build(force: bool = False) -> str:
    """Compile gemm_ref.c with gcc (OpenMP) next to this file."""
    src = os.path.join(_HERE, "gemm_ref.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", src, "-o", _LIB_PATH])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        p = ctypes.c_void_p
        i64 = ctypes.c_int64
        lib.ref_gemm_bf16_f64.argtypes = [p, p, p, i64, i64, i64, ctypes.c_int]
        lib.ref_gemm_bf16_f64.restype = None
        lib.ref_gemm_bf16_f64_elems.argtypes = [p, p, i64, i64, i64, p, p, i64, p]
        lib.ref_gemm_bf16_f64_elems.restype = None
        lib.ref_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().ref_num_threads())


def _chk(bits: np.ndarray, rows: int, cols: int) -> np.ndarray:
    a = np.ascontiguousarray(bits, dtype=np.uint16)
    assert a.shape == (rows, cols), (a.shape, rows, cols)
    return a


def gemm(a_bits: np.ndarray, b_bits: np.ndarray, threads: int = 0) -> np.ndarray:
    """Full fp64 product of two bf16-bit-pattern matrices."""
    M, K = a_bits.shape
    K2, N = b_bits.shape
    assert K == K2
    a, b = _chk(a_bits, M, K), _chk(b_bits, K, N)
    c = np.empty((M, N), dtype=np.float64)
    _load().ref_gemm_bf16_f64(a.ctypes.data, b.ctypes.data, c.ctypes.data, M, N, K, threads)
    return c


def gemm_elems(a_bits: np.ndarray, b_bits: np.ndarray, ii, jj) -> np.ndarray:
    """fp64 values of the selected elements (ii[e], jj[e])."""
    M, K = a_bits.shape
    K2, N = b_bits.shape
    assert K == K2
    a, b = _chk(a_bits, M, K), _chk(b_bits, K, N)
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    assert ii.shape == jj.shape and ii.ndim == 1
    assert ii.size == 0 or (ii.min() >= 0 and ii.max() < M and jj.min() >= 0 and jj.max() < N)
    out = np.empty(ii.size, dtype=np.float64)
    _load().ref_gemm_bf16_f64_elems(a.ctypes.data, b.ctypes.data, M, N, K, ii.ctypes.data, jj.ctypes.data,
                                    ii.size, out.ctypes.data)
    return out


def _widen(h: int) -> float:
    return struct.unpack("<f", struct.pack("<I", (int(h) & 0xFFFF) << 16))[0]


def gemm_tiny(a_bits, b_bits) -> list[list[float]]:
    """The definition as three Python loops (Python floats are fp64). Small inputs only."""
    M, K = len(a_bits), len(a_bits[0])
    N = len(b_bits[0])
    c = [[0.0] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            s = 0.0
            for k in range(K):
                s += _widen(a_bits[i][k]) * _widen(b_bits[k][j])
            c[i][j] = s
    return c


def within_tolerance(c_gpu_f64: np.ndarray, c_ref: np.ndarray) -> np.ndarray:
    """Element-wise acceptance mask."""
    return np.abs(c_gpu_f64 - c_ref) <= RTOL * np.abs(c_ref) + ATOL
