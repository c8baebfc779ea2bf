"""Pins for the row softmax / layer normalisation oracle: closed forms, invariants, independent library
routines and plain loops, chosen so that a dropped max subtraction, an unbiased variance, a misplaced
eps or a gamma/beta indexed along the wrong axis fails at least one of them."""
import math

import numpy as np
import pytest

import seeded_inputs as si
from oracle import rowwise_ref as rw


def bits(x):
    return si.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_widen_is_exact():
    vals = np.array([0.0, 1.0, -2.5, 0.0078125, 3.0e38, -1.0e-38], dtype=np.float32)
    b = bits(vals)
    assert np.array_equal(rw.widen(b), si.bf16_bits_to_f64(b))
    assert rw.widen(np.array([0x3F80, 0xC020], dtype=np.uint16)).tolist() == [1.0, -2.5]


def test_softmax_closed_forms():
    y = rw.softmax(bits([[0.0, 0.0, 0.0, 0.0], [2.0, 3.0, 2.0, 3.0]]))
    assert np.allclose(y[0], 0.25, rtol=0, atol=1e-15)
    e = math.e
    assert np.allclose(y[1], [0.5 / (1 + e), 0.5 * e / (1 + e)] * 2, rtol=1e-14)
    # one dominant entry: everything else is exp(-gap)
    y = rw.softmax(bits([[16.0, 0.0, 0.0]]))
    assert y[0, 1] == pytest.approx(math.exp(-16) / (1 + 2 * math.exp(-16)), rel=1e-14)


def test_softmax_invariants_and_large_values():
    x = si.matrix_bf16(11, 0, 6, 40, "normal", 4.0)
    y = rw.softmax(x)
    assert np.allclose(y.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    assert (y > 0).all() and (np.argmax(y, axis=1) == np.argmax(rw.widen(x), axis=1)).all()
    # shift invariance with an exactly representable shift on small integers
    xi = si.small_int_matrix_bf16(5, 0, 4, 16, -3, 3)
    shifted = bits(rw.widen(xi) + 64.0)
    assert np.allclose(rw.softmax(xi), rw.softmax(shifted), rtol=1e-14, atol=0)
    # values whose exponential overflows fp64 unless the row maximum is subtracted first
    y = rw.softmax(bits([[1000.0, 1000.0, 992.0]]))
    assert np.isfinite(y).all() and y[0, 0] == pytest.approx(1 / (2 + math.exp(-8)), rel=1e-14)
    # rows are independent: permuting rows permutes results
    assert np.array_equal(rw.softmax(x[::-1]), rw.softmax(x)[::-1])


def test_softmax_against_independent_routines():
    from scipy.special import softmax as sp_softmax
    import torch
    x = si.matrix_bf16(12, 0, 7, 33, "normal", 3.0)
    xf = si.bf16_bits_to_f64(x)
    y = rw.softmax(x)
    assert np.allclose(y, sp_softmax(xf, axis=1), rtol=1e-13, atol=0)
    assert np.allclose(y, torch.softmax(torch.from_numpy(xf), dim=1).numpy(), rtol=1e-13, atol=0)
    assert np.allclose(np.array(rw.softmax_loops(xf[:3].tolist())), y[:3], rtol=1e-13, atol=0)


def test_layernorm_closed_forms():
    one, zero = bits(np.ones(4)), bits(np.zeros(4))
    y = rw.layernorm(bits([[1.0, 2.0, 3.0, 4.0]]), one, zero, 0.0)
    # mean 2.5, biased variance 1.25 (the unbiased 5/3 would give other values)
    assert np.allclose(y[0], (np.array([1, 2, 3, 4]) - 2.5) / math.sqrt(1.25), rtol=1e-15)
    eps = 0.75
    y = rw.layernorm(bits([[1.0, 2.0, 3.0, 4.0]]), one, zero, eps)
    assert np.allclose(y[0], (np.array([1, 2, 3, 4]) - 2.5) / math.sqrt(2.0), rtol=1e-15)   # eps inside the root
    # gamma and beta run along the columns
    g, b = bits([1.0, 2.0, 4.0, 8.0]), bits([0.5, -0.5, 0.25, 0.0])
    y = rw.layernorm(bits([[-1.0, 1.0, -1.0, 1.0], [3.0, 5.0, 3.0, 5.0]]), g, b, 0.0)
    assert np.allclose(y, [[-0.5, 1.5, -3.75, 8.0]] * 2, rtol=1e-15)


def test_layernorm_invariants():
    M, N, eps = 5, 48, 1e-5
    x = si.matrix_bf16(13, 0, M, N, "normal", 2.0)
    one, zero = bits(np.ones(N)), bits(np.zeros(N))
    y = rw.layernorm(x, one, zero, eps)
    xf = si.bf16_bits_to_f64(x)
    var = xf.var(axis=1)
    assert np.allclose(y.mean(axis=1), 0.0, atol=1e-14)
    assert np.allclose((y * y).mean(axis=1), var / (var + eps), rtol=1e-12)
    # affine input change x -> 4x + 32 leaves the normalised row unchanged when eps = 0 (both exact in bf16 here)
    xi = si.small_int_matrix_bf16(6, 0, 3, 16, -3, 3)
    xi[:, 0] = bits([3.0])[0]; xi[:, 1] = bits([-3.0])[0]                     # no constant row
    o16, z16 = bits(np.ones(16)), bits(np.zeros(16))
    assert np.allclose(rw.layernorm(xi, o16, z16, 0.0), rw.layernorm(bits(4 * rw.widen(xi) + 32), o16, z16, 0.0), rtol=1e-13)


def test_layernorm_against_independent_routines():
    import torch
    M, N, eps = 6, 40, 1e-5
    x = si.matrix_bf16(14, 0, M, N, "normal", 1.5)
    g = si.matrix_bf16(14, 1, 1, N, "uniform")[0]
    b = si.matrix_bf16(14, 2, 1, N, "uniform")[0]
    y = rw.layernorm(x, g, b, eps)
    t = torch.nn.functional.layer_norm(torch.from_numpy(si.bf16_bits_to_f64(x)), (N,), torch.from_numpy(si.bf16_bits_to_f64(g)),
                                       torch.from_numpy(si.bf16_bits_to_f64(b)), eps)
    assert np.allclose(y, t.numpy(), rtol=1e-12, atol=1e-14)
    loops = rw.layernorm_loops(si.bf16_bits_to_f64(x[:2]).tolist(), si.bf16_bits_to_f64(g).tolist(),
                               si.bf16_bits_to_f64(b).tolist(), eps)
    assert np.allclose(y[:2], loops, rtol=1e-12, atol=1e-14)


def test_tolerances_admit_a_correctly_rounded_result_and_reject_small_errors():
    x = si.matrix_bf16(15, 0, 8, 256, "normal", 2.0)
    ref = rw.softmax(x)
    rounded = si.bf16_bits_to_f64(si.f32_to_bf16_bits(ref.astype(np.float32)))
    assert (np.abs(rounded - ref) <= rw.softmax_bound(ref)).all()
    assert not (np.abs(rounded * 1.02 - ref) <= rw.softmax_bound(ref)).all()
    g = si.matrix_bf16(15, 1, 1, 256, "uniform")[0]
    b = si.matrix_bf16(15, 2, 1, 256, "uniform")[0]
    ref = rw.layernorm(x, g, b, 1e-5)
    rounded = si.bf16_bits_to_f64(si.f32_to_bf16_bits(ref.astype(np.float32)))
    bound = rw.layernorm_bound(x, g, b, 1e-5)
    assert (np.abs(rounded - ref) <= bound).all()
    assert not (np.abs(rounded + 0.01 - ref) <= bound).all()
