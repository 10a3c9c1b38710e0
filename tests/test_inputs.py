"""The synthetic input generator: addressable, seeded, and of the stated distributions."""
import numpy as np

import moe_inputs as mi


def test_elements_are_addressable_and_seeded():
    a = mi.normal_f32(3, mi.STREAM_X, 0, 5000, 1.0)
    b = mi.normal_f32(3, mi.STREAM_X, 1234, 100, 1.0)
    assert np.array_equal(a[1234:1334], b)
    assert not np.array_equal(a, mi.normal_f32(4, mi.STREAM_X, 0, 5000, 1.0))
    assert not np.array_equal(a, mi.normal_f32(3, mi.STREAM_W_GATE, 0, 5000, 1.0))


def test_distribution_is_close_to_normal():
    v = mi.normal_f32(0, mi.STREAM_X, 0, 1 << 20, 2.0).astype(np.float64)
    assert abs(v.mean()) < 0.01
    assert abs(v.std() - 2.0) < 0.01
    z = v / 2.0
    assert abs(np.mean(np.abs(z) < 1.0) - 0.6827) < 0.005
    assert abs(np.mean(np.abs(z) < 2.0) - 0.9545) < 0.003
    assert abs(np.mean(z ** 4) - 3.0) < 0.15               # kurtosis of a twelve-uniform sum is 2.9


def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -3.0], np.float32)
    bits = mi.f32_to_bf16_bits(f)
    back = mi.bf16_bits_to_f32(bits)
    assert list(back) == [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7, -3.0]


def test_tensor_slices_match_whole_tensor():
    cfg = mi.small_variant(mi.CONFIGS["gptoss"], N=16, H=64, F=32)
    full = mi.host_tensor(cfg, mi.STREAM_W_DOWN)
    assert full.shape == (cfg.E, cfg.H, cfg.F) and full.dtype == np.uint16
    part = mi.host_tensor(cfg, mi.STREAM_W_DOWN, 5, 3)
    assert np.array_equal(part, full[5:8])
    w = mi.bf16_bits_to_f32(full).astype(np.float64)
    assert abs(w.std() * np.sqrt(cfg.F) - 1.0) < 0.02        # N(0, 1/fan_in)


def test_popularity_and_bias():
    cfg = mi.CONFIGS["dsv3_ep"]
    p = mi.popularity(cfg)
    assert np.isclose(p.sum(), 1.0) and p.size == 256
    ps = np.sort(p)[::-1]
    assert np.allclose(ps / ps[0], np.arange(1, 257) ** -1.2)
    b = mi.router_bias(cfg)
    assert b.dtype == np.float32 and b.max() == 0.0
    assert mi.router_bias(mi.CONFIGS["mixtral"]) is None
    c = mi.recv_segment_counts(cfg, 65536, 0)
    assert c.sum() == 65536 and c.size == 8
    q = p[:8] / p[:8].sum()
    assert np.all(np.abs(c / 65536 - q) < 0.01)
