"""Seeded input generators: determinism, bf16 rounding, label distributions, shard tables."""
import numpy as np
import pytest
import torch

from paper_2011_09208_amd import inputs


def test_bf16_rounding_matches_torch():
    r = np.random.Generator(np.random.PCG64(0))
    a = np.concatenate([
        r.standard_normal(20000).astype(np.float32) * np.float32(3.0),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0078125, 1.01171875, 3.3895314e38, 1e-40, np.inf, -np.inf],
                 dtype=np.float32),
    ])
    bits = inputs.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = inputs.bf16_bits_to_f64(bits)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy())
    assert np.isnan(inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(np.array([np.nan], np.float32))))[0]


def test_determinism_and_ranges():
    a = inputs.make_config("cfg1")
    b = inputs.make_config("cfg1")
    assert np.array_equal(a.X_bits, b.X_bits) and np.array_equal(a.W_bits, b.W_bits)
    assert np.array_equal(a.labels, b.labels)
    c = inputs.make_config("cfg1", seed=1)
    assert not np.array_equal(a.X_bits, c.X_bits)
    assert a.X_bits.shape == (32, 256) and a.W_bits.shape == (1000, 256) and a.labels.dtype == np.int32
    assert a.labels.min() >= 0 and a.labels.max() < 1000
    assert abs(inputs.bf16_bits_to_f64(a.W_bits).std() - 0.02) < 1e-3
    assert a.shards == [(0, 500), (500, 500)]


def test_w_rows_prefix_keeps_stream():
    full = inputs.make_inputs("t", 8, 16, 20000, shards=None)
    part = inputs.make_inputs("t", 8, 16, 20000, w_rows=9000)
    assert np.array_equal(part.W_bits, full.W_bits[:9000])
    assert np.array_equal(part.labels, full.labels)


def test_relu_features_nonnegative():
    p = inputs.make_inputs("t", 64, 128, 10, x_relu=True)
    x = inputs.bf16_bits_to_f64(p.X_bits)
    assert x.min() == 0.0 and 0.4 < (x == 0).mean() < 0.6


@pytest.mark.parametrize("name", list(inputs.CONFIGS))
def test_shard_tables_tile_the_classes(name):
    cfg = inputs.CONFIGS[name]
    o = 0
    for off, w in cfg["shards"]:
        assert off == o and w > 0
        o += w
    assert o == cfg["C"]


def test_uneven_partition_is_three_to_one():
    # two fast and two slow devices at 3:1 computing capacity (Section 3.3.1, initial load ratios)
    widths = [w for _, w in inputs.CONFIGS["cfg4"]["shards"]]
    assert widths == [37_500, 12_500, 37_500, 12_500]
    assert widths[0] / (widths[0] + widths[1]) == 0.75


def test_zipf_mass():
    p = inputs.zipf_probabilities(100_000, 1.1)
    assert abs(p.sum() - 1) < 1e-12 and np.all(np.diff(p) < 0)
    assert 0.94 < p[:37_500].sum() < 0.97
    p = inputs.zipf_probabilities(400_000, 1.0)
    assert 0.83 < p[:50_000].sum() < 0.86
    y = inputs.draw_labels(np.random.Generator(np.random.PCG64(0)), 4096, 100_000, ("zipf", 1.1))
    assert y.dtype == np.int32 and (y < 37_500).mean() > 0.9
