"""GPU parity of the row softmax / layer normalisation entry points (through the C ABI) against the fp64 oracle."""
import numpy as np
import pytest

import seeded_inputs as si
from oracle import rowwise_ref as rw

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

NEG_INF = np.uint16(0xFF80)          # bfloat16 -inf


@pytest.fixture(scope="module")
def swz():
    import paper_2508_20258_amd as m
    assert torch.cuda.is_available()
    return m


def to_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


SHAPES = [(1, 8, 1), (3, 40, 5), (17, 1000, 1), (17, 1000, 3), (17, 1000, 8), (64, 4096, 8), (5, 72, 4),
          (9, 8200, 7), (2, 262144, 16), (300, 2048, 2), (1031, 264, 3),
          # one workgroup per row: a row per wave (N <= 2048), rows kept in registers (N <= 32768), rows streamed twice
          (7, 2048, 1), (65, 1000, 1), (33, 2056, 1), (12, 8192, 1), (5, 32768, 1), (3, 32776, 1), (2, 100000, 1)]


def run_all_modes(fn, M, N):
    outs = []
    for mode in range(4):
        out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        fn(out, mode)
        torch.cuda.synchronize()
        outs.append(to_bits(out))
    for o in outs[1:]:
        assert np.array_equal(o, outs[0]), "result bits depend on the mode"
    return outs[0]


@pytest.mark.parametrize("M,N,chunks", SHAPES)
@pytest.mark.parametrize("scale", [1.0, 6.0])
def test_softmax_matches_oracle_in_every_mode(swz, M, N, chunks, scale):
    x = si.matrix_bf16(700 + N, 0, M, N, "normal", scale)
    if N >= 40:
        x[0, 3:N:7] = NEG_INF                       # masked entries
        x[M - 1, :N - 1] = NEG_INF                  # a row with a single finite entry
    xd = to_dev(x)
    got = run_all_modes(lambda out, mode: swz.softmax(xd, out, chunks=chunks, mode=mode), M, N)
    ref = rw.softmax(x)
    err = np.abs(si.bf16_bits_to_f64(got) - ref)
    ok = err <= rw.softmax_bound(ref)
    assert ok.all(), f"{np.count_nonzero(~ok)} of {ok.size} outside tolerance, worst {err.max()}"
    # the result does not depend on num_xcd / group_m, nor (with 256 threads per row) on how the row is cut
    one = swz.softmax(xd, chunks=1, mode=0)
    odd = swz.softmax(xd, chunks=chunks, mode=2, num_xcd=3, group_m=7)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(odd), got)
    if N > 2048:
        assert np.array_equal(to_bits(one), got)
    else:
        assert (np.abs(si.bf16_bits_to_f64(to_bits(one)) - ref) <= rw.softmax_bound(ref)).all()


@pytest.mark.parametrize("M,N,chunks", SHAPES)
@pytest.mark.parametrize("offset", [0.0, 200.0])
def test_layernorm_matches_oracle_in_every_mode(swz, M, N, chunks, offset):
    eps = 1e-5
    x = si.f32_to_bf16_bits((si.bf16_bits_to_f64(si.matrix_bf16(800 + N, 0, M, N, "normal", 2.0)) + offset).astype(np.float32))
    g = si.matrix_bf16(800 + N, 1, 1, N, "uniform", 2.0)[0]
    b = si.matrix_bf16(800 + N, 2, 1, N, "uniform")[0]
    xd, gd, bd = to_dev(x), to_dev(g), to_dev(b)
    got = run_all_modes(lambda out, mode: swz.layernorm(xd, gd, bd, out, eps=eps, chunks=chunks, mode=mode), M, N)
    ref = rw.layernorm(x, g, b, eps)
    err = np.abs(si.bf16_bits_to_f64(got) - ref)
    ok = err <= rw.layernorm_bound(x, g, b, eps)
    assert ok.all(), f"{np.count_nonzero(~ok)} of {ok.size} outside tolerance, worst {err.max()}"
    one = swz.layernorm(xd, gd, bd, eps=eps, chunks=1, mode=0)
    odd = swz.layernorm(xd, gd, bd, eps=eps, chunks=chunks, mode=2, num_xcd=3, group_m=7)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(odd), got)
    if N > 2048:
        assert np.array_equal(to_bits(one), got)
    else:
        assert (np.abs(si.bf16_bits_to_f64(to_bits(one)) - ref) <= rw.layernorm_bound(x, g, b, eps)).all()


def test_layernorm_constant_and_exact_rows(swz):
    # a constant row has variance 0: y = beta; rows of +-1 with gamma = 1, beta = 0, eps = 0 come back unchanged
    N = 512
    x = np.empty((2, N), dtype=np.float32)
    x[0] = 3.0
    x[1] = np.where(np.arange(N) % 2 == 0, -1.0, 1.0)
    xd = to_dev(si.f32_to_bf16_bits(x))
    g = torch.ones(N, dtype=torch.bfloat16, device="cuda")
    b = torch.full((N,), 0.5, dtype=torch.bfloat16, device="cuda")
    y = swz.layernorm(xd, g, b, eps=1e-5, chunks=2, mode=1).float().cpu().numpy()
    assert (y[0] == 0.5).all()
    y = swz.layernorm(xd, g, torch.zeros_like(b), eps=0.0, chunks=2, mode=1).float().cpu().numpy()
    assert np.array_equal(y[1], x[1])


def test_rowwise_full_size_in_the_measured_configuration(swz):
    # the shape and launch the profiling harness times: 8192 x 8192, 8 chunks per row; oracle on sampled rows
    M = N = 8192
    x = si.matrix_bf16(31, 0, M, N, "normal", 2.0)
    g = si.matrix_bf16(31, 1, 1, N, "uniform", 2.0)[0]
    b = si.matrix_bf16(31, 2, 1, N, "uniform")[0]
    xd, gd, bd = to_dev(x), to_dev(g), to_dev(b)
    rows = np.unique(np.concatenate([[0, 1, 7, 8, M - 1], (np.arange(64) * 2654435761 % M)]))
    sm = {mode: to_bits(swz.softmax(xd, chunks=8, mode=mode)) for mode in (0, 1)}
    ln = {mode: to_bits(swz.layernorm(xd, gd, bd, eps=1e-5, chunks=8, mode=mode)) for mode in (0, 1)}
    torch.cuda.synchronize()
    assert np.array_equal(sm[0], sm[1]) and np.array_equal(ln[0], ln[1])
    ref = rw.softmax(x[rows])
    assert (np.abs(si.bf16_bits_to_f64(sm[1][rows]) - ref) <= rw.softmax_bound(ref)).all()
    ref = rw.layernorm(x[rows], g, b, 1e-5)
    assert (np.abs(si.bf16_bits_to_f64(ln[1][rows]) - ref) <= rw.layernorm_bound(x[rows], g, b, 1e-5)).all()
    # properties that hold for every row: probabilities sum to 1 within the output rounding
    sums = si.bf16_bits_to_f64(sm[1]).sum(axis=1)
    assert np.abs(sums - 1.0).max() < 2e-3


def test_rowwise_error_paths(swz):
    x = to_dev(si.matrix_bf16(1, 0, 16, 64, "uniform"))
    y = torch.full((16, 64), 2.0, dtype=torch.bfloat16, device="cuda")
    g = torch.ones(64, dtype=torch.bfloat16, device="cuda")
    L = swz.lib
    s = torch.cuda.current_stream().cuda_stream
    xp, yp, gp = x.data_ptr(), y.data_ptr(), g.data_ptr()
    assert L.swz_softmax(xp, yp, 16, 64, 0, 0, None, s) == -1          # chunks < 1
    assert L.swz_softmax(xp, yp, 16, 64, 9, 0, None, s) == -1          # more chunks than 16-byte vectors
    assert L.swz_softmax(xp, yp, 16, 60, 1, 0, None, s) == -2          # N % 8
    assert L.swz_softmax(xp, yp, 16, 64, 1, 8, None, s) == -1          # mode
    assert L.swz_softmax(xp, yp, 16, 64, 1, 5, None, s) == -2          # skewed modes would pull a row's chunks apart: not offered
    assert L.swz_layernorm(xp, gp, gp, yp, 16, 64, 1e-5, 1, 6, None, s) == -2
    assert L.swz_softmax(None, yp, 16, 64, 1, 0, None, s) == -1
    assert L.swz_softmax(xp + 2, yp, 16, 56, 1, 0, None, s) == -2      # alignment
    assert L.swz_softmax(xp, yp, 1 << 28, 64, 8, 0, None, s) == -3     # M * chunks
    assert L.swz_layernorm(xp, None, gp, yp, 16, 64, 1e-5, 1, 0, None, s) == -1
    assert L.swz_layernorm(xp, gp, gp, yp, 16, 64, -1.0, 1, 0, None, s) == -1
    assert L.swz_layernorm(xp, gp, gp, yp, 16, 64, float("nan"), 1, 0, None, s) == -1
    assert L.swz_layernorm(xp, gp, gp, yp, 16, 1 << 25, 1e-5, 1, 0, None, s) == -2
    torch.cuda.synchronize()
    assert (y == 2.0).all()
