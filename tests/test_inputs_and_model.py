"""The seeded generator and the panel-count model."""
import numpy as np
import torch

import seeded_inputs as si
from oracle import l2_model
from oracle import pid_map as opm


def test_bf16_rounding_matches_torch_round_to_nearest_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 100000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], dtype=np.float32)]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(si.f32_to_bf16_bits(x), want)
    back = si.bf16_bits_to_f64(want)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy())


def test_generator_is_counter_based_and_seeded():
    a = si.matrix_bf16(3, 0, 40, 50, "normal", 0.5, chunk=64)
    b = si.matrix_bf16(3, 0, 40, 50, "normal", 0.5, chunk=1 << 20)
    assert np.array_equal(a, b)                                   # chunking never changes a value
    assert not np.array_equal(a, si.matrix_bf16(4, 0, 40, 50, "normal", 0.5))
    assert not np.array_equal(a, si.matrix_bf16(3, 1, 40, 50, "normal", 0.5))


def test_distributions():
    u = si.bf16_bits_to_f64(si.matrix_bf16(0, 0, 512, 512, "uniform"))
    assert -1.0 <= u.min() and u.max() <= 1.0
    assert abs(u.mean()) < 0.01 and abs(u.var() - 1 / 3) < 0.01
    n = si.bf16_bits_to_f64(si.matrix_bf16(1, 0, 512, 512, "normal", 1 / 64))
    assert abs(n.mean()) < 1e-3 and abs(n.std() * 64 - 1) < 0.02
    k = si.bf16_bits_to_f64(si.small_int_matrix_bf16(2, 0, 64, 64, -1, 1))
    assert set(np.unique(k)) == {-1.0, 0.0, 1.0}


def test_configs_have_the_stated_shapes():
    c = si.CONFIGS
    assert (c["cfg2_4096"]["M"], c["cfg2_4096"]["tile"]) == (4096, (256, 256, 64))
    assert (c["cfg5_ragged"]["M"], c["cfg5_ragged"]["N"], c["cfg5_ragged"]["K"]) == (10000, 7000, 4096)
    a, b = si.config_inputs("cfg1_512")
    assert a.shape == (512, 512) and b.shape == (512, 512) and a.dtype == np.uint16


def test_panel_model_closed_forms():
    # 32 co-resident tiles forming a 4 x 8 block touch 4 + 8 panels for 64 requests
    block = [pm * 8 + pn for pm in range(4) for pn in range(8)]
    assert abs(l2_model.predicted_hit_rate(block, 8, 1, 32) - (1 - 12 / 64)) < 1e-12
    # one tile at a time: nothing is shared
    assert l2_model.predicted_hit_rate(block, 8, 1, 1) == 0.0
    # a full row of 32 tiles shares its A panel only
    row = list(range(32))
    assert abs(l2_model.predicted_hit_rate(row, 32, 1, 32) - (1 - 33 / 64)) < 1e-12


def test_panel_model_orders_the_mappings_as_the_paper_argues():
    # skinny grid (64 x 8): round-robin gives each XCD one tile column -> worst; the swizzle fixes it
    maps = {m: opm.pid_map(64, 8, 8, 4, m) for m in range(4)}
    rate = {m: l2_model.predicted_hit_rate(maps[m], 8, 8, 32) for m in maps}
    assert rate[0] < rate[1] and rate[0] < rate[2]
    assert abs(rate[2] - (1 - 12 / 64)) < 1e-12
    # square 16 x 16 grid: only the grouped raster on top of the XCD renumbering helps
    r16 = {m: l2_model.predicted_hit_rate(opm.pid_map(16, 16, 8, 4, m), 16, 8, 32) for m in range(4)}
    assert r16[2] > r16[0] and abs(r16[1] - r16[0]) < 1e-12
