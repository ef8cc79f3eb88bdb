"""Host tests of the seeded input generator (no method arithmetic lives there)."""
import numpy as np
import pytest

from paper_2510_04286_amd import workload as wl


def test_configs_match_the_benchmark_table():
    rows = {  # name: (T, d, S, ds, E, k, He, Ns, Na)
        "tiny": (512, 256, 4, 64, 8, 2, 256, 2048, 4096),
        "lm": (4096, 512, 8, 64, 16, 2, 256, 32768, 65536),
        "headline": (16384, 1024, 16, 64, 32, 2, 256, 262144, 524288),
        "skewed": (16384, 1024, 16, 64, 32, 2, 256, 262144, 524288),
        "large": (65536, 4096, 32, 128, 64, 2, 512, 2097152, 4194304),
    }
    for name, (T, d, S, ds, E, k, He, Ns, Na) in rows.items():
        c = wl.CONFIGS[name]
        assert (c.T, c.d, c.S, c.ds, c.E, c.k, c.He, c.Ns, c.Na) == (T, d, S, ds, E, k, He, Ns, Na)
        assert c.Hr == 256
    assert wl.CONFIGS["tiny"].dtype == "f32" and wl.CONFIGS["headline"].dtype == "bf16"
    assert wl.CONFIGS["skewed"].capacity() == 20480 and wl.CONFIGS["headline"].capacity() == -1


def test_counter_based_generation_is_order_independent():
    a = wl.uniform01(7, 3, 0, 1000)
    b = np.concatenate([wl.uniform01(7, 3, 0, 400), wl.uniform01(7, 3, 400, 600)])
    np.testing.assert_array_equal(a, b)
    assert not np.array_equal(a, wl.uniform01(8, 3, 0, 1000))
    assert not np.array_equal(a, wl.uniform01(7, 4, 0, 1000))
    cfg = wl.CONFIGS["lm"].scaled(64)
    np.testing.assert_array_equal(wl.make_h(cfg)[10:20], wl.make_h(cfg, t0=10, t1=20))


def test_distributions():
    u = wl.uniform01(1, 1, 0, 200000)
    assert 0 <= u.min() and u.max() < 1 and abs(u.mean() - 0.5) < 5e-3 and abs(u.var() - 1 / 12) < 2e-3
    z = wl.normal(1, 2, 0, 200000)
    assert abs(z.mean()) < 1e-2 and abs(z.std() - 1) < 1e-2 and abs((z ** 3).mean()) < 3e-2
    assert abs((z ** 4).mean() - 3) < 0.1


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -9, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -9, -1.0 - 2 ** -9, 3.14159], np.float32)
    r = wl.round_to_bf16(x)
    # bf16 spacing at 1 is 2^-7: 1+2^-9 rounds down, 1+2^-8 is a tie -> even (1.0), 1+3*2^-9 rounds up
    np.testing.assert_array_equal(r[:3], [1.0, 1.0, 1.0])
    assert r[3] == np.float32(1.0 + 2 ** -7) and r[4] == np.float32(-1.0)
    np.testing.assert_array_equal(wl.bf16_bits_to_f32(wl.bf16_bits(r)), r)
    tie_up = np.array([1.0 + 2 ** -7 + 2 ** -8], np.float32)  # tie between odd 1+2^-7 and even 1+2^-6
    assert wl.round_to_bf16(tie_up)[0] == np.float32(1.0 + 2 ** -6)
    rng = np.random.default_rng(0)
    y = rng.normal(0, 1, 10000).astype(np.float32)
    ry = wl.round_to_bf16(y)
    assert np.all(np.abs(ry - y) <= np.abs(y) * 2 ** -8)
    with pytest.raises(AssertionError):
        wl.bf16_bits(np.array([3.14159], np.float32))


def test_weights_follow_linear_default_init():
    cfg = wl.CONFIGS["headline"].scaled(8)
    w = wl.make_weights(cfg)
    assert w["Wr1"].shape == (64, 256) and w["Wr2"].shape == (256, 32) and w["br2"].shape == (32,)
    assert w["W1"].shape == (32, 64, 256) and w["W2"].shape == (32, 256, 64) and w["b2"].shape == (32, 64)
    for name, fan_in in [("Wr1", 64), ("br1", 64), ("Wr2", 256), ("W1", 64), ("b1", 64), ("W2", 256), ("b2", 256)]:
        b = 1 / np.sqrt(fan_in)
        assert np.abs(w[name]).max() <= b * (1 + 2 ** -8)
        assert np.abs(w[name]).max() > 0.9 * b or w[name].size < 64
        wl.bf16_bits(w[name])  # representable
    assert abs(w["W1"].mean()) < 1e-3


def test_layernorm_recipe_and_tiny_dtype():
    cfg = wl.CONFIGS["lm"].scaled(32)
    h = wl.make_h(cfg).astype(np.float64)
    assert np.all(np.abs(h.mean(axis=1)) < 2e-3) and np.all(np.abs(h.var(axis=1) - 1) < 1e-2)
    t = wl.make_h(wl.CONFIGS["tiny"])
    assert t.dtype == np.float32 and np.any(t.view(np.uint32) & 0xFFFF)  # fp32 storage keeps low bits


def test_random_topk_tables():
    idx = wl.make_topk_idx(5000, 3, 16, seed=3)
    assert idx.dtype == np.int32 and idx.shape == (5000, 3) and idx.min() >= 0 and idx.max() < 16
    assert all(len(set(r)) == 3 for r in idx[:200])
    skew = wl.make_topk_idx(20000, 2, 32, seed=4, zipf_s=1.2)
    c = np.bincount(skew.reshape(-1), minlength=32)
    assert c[0] > 3 * c[8] > 0
