"""Host model of the arithmetic the int8 kernels' output stage uses on its fast path (clamp on the way in, then either
an fp32 fused multiply-add with the constant 1.5 * 2^23 or an integer rounding shift), checked against the oracle's
scale-down / saturate / ReLU (Appendix C, Figs. 14-15) on the values where it could go wrong: the clamp bounds, every
tie beside them, the ends of int32, and random sums.  The GPU tests run the kernels themselves on the same values."""
import numpy as np
import pytest

import oracle


def bounds(shift, act):
    rnd = (1 << (shift - 1)) - 1
    return (0 if act else -128 * (1 << shift)), (127 << shift) + rnd, rnd


def model_float(t, shift, act):
    """convert, clamp as fp32, one fused multiply-add (computed exactly in float64, rounded once to fp32); the low
    byte of the bit pattern is the output."""
    lo, hi, _ = bounds(shift, act)
    assert float(np.float32(lo)) == lo and float(np.float32(hi)) == hi  # exact bounds: the premise of the path
    c = np.clip(t.astype(np.int32).astype(np.float32), np.float32(lo), np.float32(hi))
    r = (c.astype(np.float64) * 2.0 ** -shift + 12582912.0).astype(np.float32)
    return (r.view(np.uint32) & 0xFF).astype(np.uint8).view(np.int8).astype(np.int64)


def model_int(t, shift, act):
    lo, hi, rnd = bounds(shift, act)
    c = np.clip(t.astype(np.int64), lo, hi)
    s = c + ((c >> shift) & 1) + rnd
    assert s.max() < 2 ** 31 and s.min() >= -(2 ** 31)  # the rounding add stays inside int32
    return s >> shift


def sums(shift):
    rng = np.random.default_rng(shift)
    half = 1 << (shift - 1)
    pts = [rng.integers(-(2 ** 31), 2 ** 31, 20000)]
    for k in list(range(-131, -124)) + list(range(-3, 4)) + list(range(124, 131)):
        pts.append((k << shift) + np.arange(-3, 4))
        pts.append((k << shift) + half + np.arange(-3, 4))
    pts.append(np.array([-(2 ** 31), 2 ** 31 - 1, -(2 ** 31) + 1, 2 ** 31 - 2, 2 ** 24, 2 ** 24 + 1, -(2 ** 24) - 1, 2 ** 30, -(2 ** 30)]))
    return np.clip(np.concatenate(pts), -(2 ** 31), 2 ** 31 - 1).astype(np.int64)


@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("shift", range(1, 24))
def test_fast_forms_equal_the_oracle(shift, act):
    t = sums(shift)
    want = np.asarray(oracle.requantise_vec(t, shift, act), dtype=np.int64)
    np.testing.assert_array_equal(model_int(t, shift, act), want)
    if shift <= 17:  # beyond 17 the bounds are not exact in fp32 and the kernels use the integer form
        np.testing.assert_array_equal(model_float(t, shift, act), want)


def test_float_form_needs_exact_bounds():
    lo, hi, _ = bounds(18, 0)
    assert float(np.float32(hi)) != hi  # 127 * 2^18 + 2^17 - 1 has 25 significant bits
