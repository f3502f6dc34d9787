"""The seeded input generator: determinism, storage formats, distribution shape."""
import numpy as np

from paper_2407_13885_amd import workloads as wl


def test_counter_based_streams_are_reproducible_and_sliceable():
    a = wl.words(7, 2, 0, 1000)
    b = wl.words(7, 2, 500, 500)
    assert np.array_equal(a[500:], b)
    assert not np.array_equal(wl.words(7, 3, 0, 16), wl.words(7, 2, 0, 16))
    assert not np.array_equal(wl.words(8, 2, 0, 16), wl.words(7, 2, 0, 16))
    assert len(np.unique(a)) == 1000


def test_normal_moments_and_uniform_range():
    z = wl.standard_normal(0, wl.STREAM_Q, 1 << 18)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01
    assert abs((z ** 3).mean()) < 0.03 and abs((z ** 4).mean() - 3.0) < 0.1
    u = wl.uniform01(0, wl.STREAM_MASK, 1 << 18)
    assert 0.0 < u.min() and u.max() < 1.0 and abs(u.mean() - 0.5) < 0.005


def test_bf16_round_to_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 (even) and 1 + 2^-7: goes to 1.0;
    # 1 + 3*2^-8 is a tie between 1 + 2^-7 (odd) and 1 + 2^-6: goes up.
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 0.0],
                 dtype=np.float32)
    b = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(b)
    assert back.tolist() == [1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5, 0.0]
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 100
    rb = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(r))
    assert (np.abs(rb - r) <= np.abs(r) * 2.0 ** -8).all()   # half an ulp of an 8-bit significand


def test_config_shapes_and_recipes():
    c1 = wl.c1()
    assert c1.Q.shape == (1, 1, 128, 64) and c1.Q.dtype == np.float32 and c1.scale == np.float32(0.125)
    assert c1.elements == 16384 and c1.algorithmic_bytes == 128 * 1024
    s = wl.c2(rows=256)
    assert s.S.shape == (256, 2048) and s.S.dtype == np.uint16
    v = wl.widen(s.S, "bf16")
    peaks = (v == 8.0).mean()
    assert 0.008 < peaks < 0.012
    assert abs(v[v != 8.0].std() - 2.0) < 0.02
    # the small matrix is a prefix of the big one (flat counter)
    assert np.array_equal(wl.c2(rows=8).S, s.S[:8])
    x = wl.fused_inputs("t", "bf16", 1, 2, 64, 16, seed=4, row_factor=(0.5, 3.0))
    rms = np.sqrt((wl.widen(x.Q, "bf16") ** 2).mean(-1))
    assert rms.min() > 0.2 and rms.max() < 5.0 and rms.std() > 0.3
