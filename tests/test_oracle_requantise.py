"""Pins for the oracle's scale-down / saturate / ReLU output stage (Appendix C, Figs. 14-15)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from conftest import read_golden_table


def test_rne_rshift_hand_values():
    for v, s, want in read_golden_table("rne_rshift_hand.txt"):
        assert oracle.rne_rshift(v, s) == want, (v, s)


def test_requantise_hand_values():
    for acc, shift, relu, want in read_golden_table("requantise_hand.txt"):
        assert oracle.requantise(acc, shift, relu) == want, (acc, shift, relu)


def test_rne_rshift_exact_rationals():
    # Python rounds an exact Fraction half-way case to the even integer.
    for s in range(0, 15):
        for v in list(range(-3000, 3001)) + [2 ** 31 - 1, -(2 ** 31), 2 ** 30, -(2 ** 30) - 1, 2 ** 31 - 1 - 2 ** 13]:
            assert oracle.rne_rshift(v, s) == round(Fraction(v, 2 ** s)), (v, s)


@pytest.mark.parametrize("s", list(range(0, 13)) + [16, 20, 31])
def test_rne_rshift_vs_float64_rint(s):
    # v / 2^s is exact in float64 for |v| < 2^53; numpy.rint rounds half to even.
    v = np.arange(-(1 << 17), (1 << 17) + 1, dtype=np.int64)
    rng = np.random.default_rng(s)
    v = np.concatenate([v, rng.integers(-(1 << 31), 1 << 31, size=200000, dtype=np.int64)])
    want = np.rint(v.astype(np.float64) / float(1 << s)).astype(np.int64)
    np.testing.assert_array_equal(oracle.rne_rshift_vec(v, s), want)


def test_rne_rshift_ties_are_even_and_monotone():
    for s in (1, 4, 8, 10):
        ties = (2 * np.arange(-50, 50, dtype=np.int64) + 1) << (s - 1)  # (odd/2) * 2^s
        out = oracle.rne_rshift_vec(ties, s)
        assert np.all(out % 2 == 0)
        assert np.all(np.abs(out * (1 << s) - ties) == (1 << (s - 1)))
        v = np.arange(-5000, 5000, dtype=np.int64)
        assert np.all(np.diff(oracle.rne_rshift_vec(v, s)) >= 0)


def test_stage_order_is_immaterial():
    # shift, saturation and ReLU are monotone maps fixing 0, so every order gives one result;
    # the oracle uses shift -> saturate -> ReLU.
    rng = np.random.default_rng(7)
    acc = np.concatenate([rng.integers(-(1 << 31), 1 << 31, size=20000, dtype=np.int64),
                          rng.integers(-70000, 70000, size=20000, dtype=np.int64)])
    for s in (0, 1, 8, 9, 10):
        sh = lambda t: oracle.rne_rshift_vec(t, s)
        # saturation bounds before the shift, expressed on the unshifted scale, lose ties; so saturate only
        # after the shift, and permute ReLU through all three positions
        sat = lambda t: np.clip(t, -128, 127)
        relu = lambda t: np.maximum(t, 0)
        base = oracle.requantise_vec(acc, s, oracle.ACT_RELU).astype(np.int64)
        np.testing.assert_array_equal(relu(sat(sh(acc))), base)
        np.testing.assert_array_equal(sat(relu(sh(acc))), base)
        np.testing.assert_array_equal(sat(sh(relu(acc))), base)
        none = oracle.requantise_vec(acc, s, oracle.ACT_NONE).astype(np.int64)
        np.testing.assert_array_equal(sat(sh(acc)), none)
        # saturating first at the pre-image of the int8 range is also equivalent
        lo, hi = -128 * (1 << s), 127 * (1 << s)
        np.testing.assert_array_equal(sh(np.clip(acc, lo, hi)), none)
