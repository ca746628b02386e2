"""Arithmetic premises that the HIP kernels rely on, checked here with numpy alone (the GPU
side checks the first one on the device itself, see rtc_selftest_half_minmax)."""
import numpy as np


def test_half_float_patterns_below_0x7c00_order_like_integers():
    """The packed 16-bit kernels reduce integers in [0, 0x7BFF] with half-float minimum / maximum
    instructions: every such bit pattern is a finite non-negative half float (denormals included)
    and the patterns order exactly like the values they encode."""
    bits = np.arange(0x7C00, dtype=np.uint16)
    vals = bits.view(np.float16).astype(np.float64)
    assert np.all(np.isfinite(vals)) and vals[0] == 0.0
    assert np.all(np.diff(vals) > 0)


def test_fp64_is_exact_on_integers_within_2_pow_51():
    """int64 pairs whose values all lie within +-2^51 run through the fp64 kernel: conversions,
    sums, differences and comparisons of such integers are exact in fp64."""
    rng = np.random.default_rng(3)
    lim = 1 << 51
    a = np.concatenate([rng.integers(-lim, lim + 1, 100000), [lim, -lim, lim, -lim, lim - 1]])
    b = np.concatenate([rng.integers(-lim, lim + 1, 100000), [lim, -lim, -lim, lim, 1]])
    fa, fb = a.astype(np.float64), b.astype(np.float64)
    assert np.array_equal(fa.astype(np.int64), a) and np.array_equal(fb.astype(np.int64), b)
    assert np.array_equal((fa + fb).astype(np.int64), a + b)
    assert np.array_equal((fa - fb).astype(np.int64), a - b)
    assert np.array_equal(fa < fb, a < b) and np.array_equal(np.minimum(fa, fb).astype(np.int64), np.minimum(a, b))


def test_low_words_carry_a_rebased_difference():
    """The re-based 32-bit items keep (value - base) as the low 32 bits of the 64-bit difference:
    whenever the true difference lies in [0, 2^31) those bits are the difference itself, whatever
    the magnitudes."""
    rng = np.random.default_rng(4)
    base = rng.integers(-(1 << 62), 1 << 62, 100000)
    diff = rng.integers(0, 1 << 31, 100000)
    low = ((base + diff).astype(np.uint64) - base.astype(np.uint64)).astype(np.uint32).astype(np.int32)
    assert np.array_equal(low.astype(np.int64), diff)
