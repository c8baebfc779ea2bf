"""fp64 reference row softmax and layer normalisation over bf16 bit patterns (test infrastructure only).

The two row-wise kernels of the paper's evaluation whose swizzle co-locates the column chunks of
one row on one XCD (SwizzlePerf, Results; Appendix "Case Study: Other Swizzling Pattern
Examples").  The swizzle changes which workgroup produces which chunk, never the values, so the
oracle is the textbook definition of each operation, written out in fp64:

    softmax    y[i][j] = exp(x[i][j] - m_i) / sum_k exp(x[i][k] - m_i),   m_i = max_k x[i][k]
    layernorm  y[i][j] = (x[i][j] - mu_i) / sqrt(var_i + eps) * gamma[j] + beta[j],
               mu_i = mean_k x[i][k],  var_i = mean_k (x[i][k] - mu_i)^2   (biased, as in the
               original layer normalisation)

Inputs are uint16 arrays of bfloat16 bit patterns (the bits the GPU gets), widened exactly.
`*_loops` are the same definitions as plain Python loops with the math module, for tiny cases.

Acceptance rule for a bf16 result computed in fp32 (every element):
    softmax    |y_gpu - y_ref| <= 2^-8 |y_ref| + 1e-30
    layernorm  |y_gpu - y_ref| <= 2^-8 |y_ref| + 1e-4 (1 + |gamma_j| |xhat_ij| + |beta_j|)
"""
from __future__ import annotations

import math

import numpy as np

SOFTMAX_RTOL = 2.0 ** -8
SOFTMAX_ATOL = 1e-30
LAYERNORM_RTOL = 2.0 ** -8
LAYERNORM_ATOL = 1e-4


def widen(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns -> float64, exactly (a bfloat16 is the top half of a float32)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def softmax(x_bits: np.ndarray) -> np.ndarray:
    x = widen(x_bits)
    m = x.max(axis=1, keepdims=True)
    e = np.exp(x - m)
    return e / e.sum(axis=1, keepdims=True)


def layernorm(x_bits: np.ndarray, gamma_bits: np.ndarray, beta_bits: np.ndarray, eps: float) -> np.ndarray:
    x, g, b = widen(x_bits), widen(gamma_bits), widen(beta_bits)
    mu = x.sum(axis=1, keepdims=True) / x.shape[1]
    d = x - mu
    var = (d * d).sum(axis=1, keepdims=True) / x.shape[1]
    return d / np.sqrt(var + eps) * g[None, :] + b[None, :]


def layernorm_bound(x_bits: np.ndarray, gamma_bits: np.ndarray, beta_bits: np.ndarray, eps: float) -> np.ndarray:
    """Per-element allowed |y_gpu - y_ref| of the acceptance rule."""
    x, g, b = widen(x_bits), widen(gamma_bits), widen(beta_bits)
    ref = layernorm(x_bits, gamma_bits, beta_bits, eps)
    mu = x.mean(axis=1, keepdims=True)
    xhat = (x - mu) / np.sqrt(((x - mu) ** 2).mean(axis=1, keepdims=True) + eps)
    return LAYERNORM_RTOL * np.abs(ref) + LAYERNORM_ATOL * (1.0 + np.abs(g)[None, :] * np.abs(xhat) + np.abs(b)[None, :])


def softmax_bound(ref: np.ndarray) -> np.ndarray:
    return SOFTMAX_RTOL * np.abs(ref) + SOFTMAX_ATOL


def softmax_loops(rows: list[list[float]]) -> list[list[float]]:
    out = []
    for row in rows:
        m = row[0]
        for v in row:
            if v > m:
                m = v
        total = 0.0
        for v in row:
            total += math.exp(v - m)
        out.append([math.exp(v - m) / total for v in row])
    return out


def layernorm_loops(rows: list[list[float]], gamma: list[float], beta: list[float], eps: float) -> list[list[float]]:
    out = []
    for row in rows:
        n = len(row)
        mu = 0.0
        for v in row:
            mu += v
        mu /= n
        var = 0.0
        for v in row:
            var += (v - mu) * (v - mu)
        var /= n
        out.append([(row[j] - mu) / math.sqrt(var + eps) * gamma[j] + beta[j] for j in range(n)])
    return out
