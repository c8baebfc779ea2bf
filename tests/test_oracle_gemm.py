"""Pins for the fp64 GEMM oracle."""
import numpy as np
import pytest

import seeded_inputs as si
from oracle import gemm_ref


def bits(x):
    return si.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_matches_three_python_loops_on_tiny_ragged_shapes():
    for seed, (M, N, K) in enumerate([(3, 5, 7), (1, 1, 1), (4, 2, 9), (6, 7, 1)]):
        a = si.matrix_bf16(seed, 0, M, K, "uniform")
        b = si.matrix_bf16(seed, 1, K, N, "normal")
        want = np.array(gemm_ref.gemm_tiny(a.tolist(), b.tolist()))
        got = gemm_ref.gemm(a, b)
        assert np.array_equal(got, want)            # same order of summation -> identical doubles


def test_matches_numpy_float64_matmul():
    # non-square, asymmetric data: a transposed operand or swapped index cannot pass
    M, N, K = 37, 53, 91
    a = si.matrix_bf16(11, 0, M, K, "normal")
    b = si.matrix_bf16(11, 1, K, N, "uniform")
    want = si.bf16_bits_to_f64(a) @ si.bf16_bits_to_f64(b)
    got = gemm_ref.gemm(a, b)
    assert got.shape == (M, N)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    # square case too, where a transposed result would still have the right shape
    a2 = si.matrix_bf16(12, 0, 40, 40, "normal")
    b2 = si.matrix_bf16(12, 1, 40, 40, "normal")
    want2 = si.bf16_bits_to_f64(a2) @ si.bf16_bits_to_f64(b2)
    np.testing.assert_allclose(gemm_ref.gemm(a2, b2), want2, rtol=1e-12, atol=1e-12)
    assert np.abs(want2 - want2.T).max() > 1.0


def test_threads_do_not_change_the_result():
    a = si.matrix_bf16(5, 0, 64, 80, "normal")
    b = si.matrix_bf16(5, 1, 80, 48, "normal")
    assert np.array_equal(gemm_ref.gemm(a, b, threads=1), gemm_ref.gemm(a, b, threads=4))


def test_closed_forms():
    K = 200
    ones_a = bits(np.ones((9, K)))
    ones_b = bits(np.ones((K, 13)))
    assert np.array_equal(gemm_ref.gemm(ones_a, ones_b), np.full((9, 13), float(K)))
    # identity B copies A; identity A copies B
    a = si.matrix_bf16(2, 0, 17, 32, "uniform")
    eye = bits(np.eye(32))
    assert np.array_equal(gemm_ref.gemm(a, eye), si.bf16_bits_to_f64(a))
    b = si.matrix_bf16(2, 1, 32, 21, "uniform")
    assert np.array_equal(gemm_ref.gemm(eye, b), si.bf16_bits_to_f64(b))
    # one-hot column selector: C[:, j] = A[:, perm[j]]
    perm = np.random.default_rng(0).permutation(32)
    sel = np.zeros((32, 32), dtype=np.float32)
    sel[perm, np.arange(32)] = 1.0
    assert np.array_equal(gemm_ref.gemm(a, bits(sel)), si.bf16_bits_to_f64(a)[:, perm])
    # rank-one: outer product of exactly representable vectors
    u = np.arange(1, 8, dtype=np.float32)[:, None]
    v = np.array([[1.0, -2.0, 0.5, 4.0]], dtype=np.float32)
    assert np.array_equal(gemm_ref.gemm(bits(u), bits(v)), (u @ v).astype(np.float64))


def test_widening_is_exact_for_every_finite_bf16_pattern():
    allbits = np.arange(65536, dtype=np.uint16)
    finite = allbits[((allbits >> 7) & 0xFF) != 0xFF].reshape(1, -1)
    one = bits(np.ones((1, 1)))
    got = gemm_ref.gemm(one, finite)                # 1 x n row of widened values
    import torch
    want = torch.from_numpy(finite.astype(np.int32).astype(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, want)


def test_selected_elements_agree_with_full_product():
    M, N, K = 50, 70, 33
    a = si.matrix_bf16(8, 0, M, K, "normal")
    b = si.matrix_bf16(8, 1, K, N, "normal")
    full = gemm_ref.gemm(a, b)
    rng = np.random.default_rng(1)
    ii = rng.integers(0, M, 500)
    jj = rng.integers(0, N, 500)
    np.testing.assert_allclose(gemm_ref.gemm_elems(a, b, ii, jj), full[ii, jj], rtol=1e-13, atol=1e-13)
    assert gemm_ref.gemm_elems(a, b, [], []).size == 0


def test_tolerance_rule():
    ref = np.array([0.0, 1.0, -100.0, 100.0])
    ok = ref + np.array([0.0099, 0.0199, 1.0, -1.009])        # bound: 0.01, 0.02, 1.01, 1.01
    bad = ref + np.array([0.0101, 0.0201, 1.02, -1.02])
    assert gemm_ref.within_tolerance(ok, ref).all()
    assert not gemm_ref.within_tolerance(bad, ref).any()


def test_bf16_output_rounding_leaves_margin_under_the_tolerance():
    # A correctly rounded bf16 result is within 2^-9 relative of the exact value: well inside 1e-2.
    a, b = si.config_inputs("cfg1_512")
    ref = gemm_ref.gemm(a[:64], b[:, :64])
    rounded = si.bf16_bits_to_f64(si.f32_to_bf16_bits(ref.astype(np.float32)))
    assert gemm_ref.within_tolerance(rounded, ref).all()
    assert (np.abs(rounded - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-30).all()


# ---------------------------------------------------------------------------- transpose oracle

def test_transpose_oracle_pins():
    from oracle import transpose_ref
    assert transpose_ref.transpose_loops([[1, 2, 3], [4, 5, 6]]) == [[1, 4], [2, 5], [3, 6]]
    x = si.matrix_bf16(3, 0, 24, 40, "uniform")
    t = transpose_ref.transpose(x)
    assert t.shape == (40, 24) and t.flags["C_CONTIGUOUS"]
    assert t.tolist() == transpose_ref.transpose_loops(x.tolist())
    assert np.array_equal(transpose_ref.transpose(t), x)                 # involution
    assert t[7, 5] == x[5, 7] and t[39, 0] == x[0, 39]


def test_transpose_oracle_moves_four_byte_elements_verbatim():
    # the definition does not care about the element width: every 32-bit pattern (NaN payloads, -0.0, denormals
    # included) must arrive bit for bit at the mirrored position
    from oracle import transpose_ref
    rng = np.random.default_rng(11)
    x = rng.integers(0, 1 << 32, size=(12, 20), dtype=np.uint64).astype(np.uint32)
    x[0, 1], x[3, 2], x[5, 19] = 0x7FC00123, 0x80000000, 0x00000001
    t = transpose_ref.transpose(x)
    assert t.dtype == np.uint32 and t.shape == (20, 12) and t.flags["C_CONTIGUOUS"]
    assert t.tolist() == transpose_ref.transpose_loops(x.tolist())
    assert t[1, 0] == 0x7FC00123 and t[2, 3] == 0x80000000 and t[19, 5] == 1
    assert np.array_equal(transpose_ref.transpose(t), x)
    # as float32 views: same bits (a value comparison would lose the NaN)
    f = x.view(np.float32)
    assert np.array_equal(transpose_ref.transpose(f).view(np.uint32), t)
