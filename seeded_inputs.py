"""Seeded synthetic GEMM inputs, shared by the tests, the benchmark and the smoke check.

This module only *draws numbers*: it holds none of the method's arithmetic (no PID maps,
no matrix products) and imports neither the CPU oracle nor the HIP library, so both can be
fed the same bits without sharing code with each other.

Generator (counter based, so any element can be produced without producing the others):

    z      = splitmix64(seed * 2^40 + matrix_id * 2^36 + stream * 2^35 + index)
    u      = (z >> 11) * 2^-53                      in [0, 1)
    U[-1,1): 2u - 1
    N(0,1) : Box-Muller, sqrt(-2 ln(1 - u0)) * cos(2 pi u1), u0/u1 from stream 0/1

Every value is then rounded to bfloat16 (round to nearest, ties to even) and returned as
its 16-bit pattern (numpy uint16), row-major.  The bit patterns are the inputs: the oracle
widens them exactly to fp64 and the GPU reads them as bf16.
"""
from __future__ import annotations

import numpy as np

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """One round of the splitmix64 output function on a uint64 array (wraps mod 2^64)."""
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def _unit(seed: int, matrix_id: int, stream: int, start: int, count: int) -> np.ndarray:
    base = (int(seed) << 40) + (int(matrix_id) << 36) + (int(stream) << 35) + int(start)
    idx = np.arange(count, dtype=np.uint64) + np.uint64(base & 0xFFFFFFFFFFFFFFFF)
    z = _splitmix64(idx)
    return (z >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> bf16 bit patterns (uint16), round to nearest even. Finite inputs only."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exact."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def matrix_bf16(seed: int, matrix_id: int, rows: int, cols: int, dist: str,
                scale: float = 1.0, chunk: int = 1 << 22) -> np.ndarray:
    """rows x cols row-major matrix of bf16 bit patterns.

    dist = "uniform": scale * U[-1,1);  dist = "normal": scale * N(0,1).
    matrix_id 0 is A, 1 is B by convention.
    """
    n = rows * cols
    out = np.empty(n, dtype=np.uint16)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        if dist == "uniform":
            v = 2.0 * _unit(seed, matrix_id, 0, s, c) - 1.0
        elif dist == "normal":
            u0 = _unit(seed, matrix_id, 0, s, c)
            u1 = _unit(seed, matrix_id, 1, s, c)
            v = np.sqrt(-2.0 * np.log1p(-u0)) * np.cos(2.0 * np.pi * u1)
        else:
            raise ValueError(f"unknown dist {dist!r}")
        out[s:s + c] = f32_to_bf16_bits((v * scale).astype(np.float32))
    return out.reshape(rows, cols)


def small_int_matrix_bf16(seed: int, matrix_id: int, rows: int, cols: int, lo: int = -1, hi: int = 1) -> np.ndarray:
    """Integer-valued matrix with entries in [lo, hi] (exactly representable in bf16)."""
    u = _unit(seed, matrix_id, 0, 0, rows * cols)
    v = np.floor(u * (hi - lo + 1)).astype(np.int64) + lo
    return f32_to_bf16_bits(v.astype(np.float32)).reshape(rows, cols)


# The five workloads: (M, N, K), value recipe for A and B, seed, tile shape.
CONFIGS = {
    "cfg1_512": dict(M=512, N=512, K=512, seed=0, a=("uniform", 1.0), b=("uniform", 1.0), tile=(128, 128, 64)),
    "cfg2_4096": dict(M=4096, N=4096, K=4096, seed=1, a=("normal", 4096 ** -0.5), b=("normal", 4096 ** -0.5), tile=(256, 256, 64)),
    "cfg3_8192": dict(M=8192, N=8192, K=8192, seed=2, a=("normal", 8192 ** -0.5), b=("normal", 8192 ** -0.5), tile=(256, 256, 64)),
    "cfg4_skinny": dict(M=16384, N=2048, K=8192, seed=3, a=("normal", 1.0), b=("normal", 0.02), tile=(256, 256, 64)),
    "cfg5_ragged": dict(M=10000, N=7000, K=4096, seed=4, a=("uniform", 1.0), b=("uniform", 1.0), tile=(256, 256, 64)),
}


def config_inputs(name: str):
    """(A_bits, B_bits) for one of CONFIGS."""
    c = CONFIGS[name]
    a = matrix_bf16(c["seed"], 0, c["M"], c["K"], c["a"][0], c["a"][1])
    b = matrix_bf16(c["seed"], 1, c["K"], c["N"], c["b"][0], c["b"][1])
    return a, b
