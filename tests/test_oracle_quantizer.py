"""Pins of the quantizer oracle (Eq. 8-10, Section 4.1) to what the paper and IEEE
arithmetic fix: the thresholds the paper states, bankers rounding at exact ties,
the two printed forms of the weight quantizer, value ranges, monotonicity, and exact
rational arithmetic where the division is exact."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import quantizer as q


def bankers(x: Fraction) -> int:
    """Round half to even on an exact rational."""
    fl = x.numerator // x.denominator
    rem = x - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def clipf(x: Fraction, lo, hi) -> Fraction:
    return min(max(x, Fraction(lo)), Fraction(hi))


def test_thresholds_stated_by_the_paper():
    # "partitioned into three levels with the quantization thresholds {-alpha1/2, alpha2/2}"
    a1, a2 = 0.8, 0.3
    p = np.array([-5.0, -0.41, -0.39, -0.1, 0.0, 0.1, 0.149, 0.151, 0.3, 7.0], np.float32)
    assert q.quantize_weight(p, a1, a2).tolist() == [-1, -1, 0, 0, 0, 0, 0, 1, 1, 1]
    # ReLU case: thresholds alpha1/2 and alpha1 + alpha2/2; values {0,1,2}
    p = np.array([-3.0, 0.0, 0.39, 0.41, 0.8, 0.94, 0.96, 50.0], np.float32)
    assert q.quantize_relu_act(p, a1, a2).tolist() == [0, 0, 0, 1, 1, 1, 2, 2]


def test_bankers_rounding_at_exact_ties():
    # step sizes that are powers of two make p / alpha exact, so +-alpha/2 is an exact tie -> 0
    a1, a2 = 0.5, 2.0
    assert q.quantize_weight(np.float32(-0.25), a1, a2) == 0      # -0.5 rounds to -0
    assert q.quantize_weight(np.float32(1.0), a1, a2) == 0        # +0.5 rounds to 0
    assert q.quantize_weight(np.nextafter(np.float32(-0.25), np.float32(-1)), a1, a2) == -1
    assert q.quantize_weight(np.nextafter(np.float32(1.0), np.float32(2)), a1, a2) == 1
    assert q.quantize_relu_act(np.float32(0.25), a1, a2) == 0     # p/alpha1 = 0.5 -> 0
    assert q.quantize_relu_act(np.float32(1.5), a1, a2) == 1      # (p-alpha1)/alpha2 = 0.5 -> 0, first term 1
    assert q.quantize_relu_act(np.nextafter(np.float32(1.5), np.float32(2)), a1, a2) == 2


def test_unified_form_equals_piecewise_form():
    rnd = np.random.default_rng(5)
    p = rnd.standard_normal(20000).astype(np.float32)
    p[:5] = [0.0, -0.0, 1e-30, -1e-30, 3.0]
    for a1, a2 in [(0.7, 0.9), (1.3, 0.2), (0.05, 2.5)]:
        assert np.array_equal(q.quantize_weight(p, a1, a2), q.quantize_weight_piecewise(p, a1, a2))


def test_value_ranges_and_monotonicity():
    rnd = np.random.default_rng(6)
    p = np.sort(rnd.standard_normal(50000).astype(np.float32) * 2)
    for a1, a2 in [(0.7, 0.9), (1.3, 0.2)]:
        w = q.quantize_weight(p, a1, a2)
        assert set(np.unique(w)) <= {-1, 0, 1} and (np.diff(w) >= 0).all()
        a = q.quantize_relu_act(p, a1, a2)
        assert set(np.unique(a)) <= {0, 1, 2} and (np.diff(a) >= 0).all()
        assert (a[p <= 0] == 0).all()
    lv = q.levels_from_floats(p, True, 0, 0.7, 0.9)
    assert set(np.unique(lv)) <= {0, 1, 2}
    assert np.array_equal(lv, q.quantize_weight(p, 0.7, 0.9) + 1)
    assert np.array_equal(q.levels_from_floats(p, False, 1, 0.7, 0.9), q.quantize_relu_act(p, 0.7, 0.9))
    assert np.array_equal(q.levels_from_floats(p, False, 0, 0.7, 0.9), lv)


@pytest.mark.parametrize("a1,a2", [(0.5, 0.25), (2.0, 0.125), (1.0, 1.0)])
def test_against_exact_rational_arithmetic(a1, a2):
    # power-of-two step sizes: float32 division and subtraction are exact, so Eq. 9 / Eq. 10 can be
    # evaluated in exact rationals with an independent round-half-to-even
    rnd = np.random.default_rng(7)
    p = (rnd.integers(-4096, 4096, size=4000) / 1024.0).astype(np.float32)      # multiples of 2^-10
    A1, A2 = Fraction(a1), Fraction(a2)
    want_w = [bankers(clipf(Fraction(float(v)) / A1, -1, 0)) + bankers(clipf(Fraction(float(v)) / A2, 0, 1)) for v in p]
    assert q.quantize_weight(p, a1, a2).tolist() == want_w
    want_a = [bankers(clipf(Fraction(float(v)) / A1, 0, 1)) + bankers(clipf((Fraction(float(v)) - A1) / A2, 0, 1))
              for v in p]
    assert q.quantize_relu_act(p, a1, a2).tolist() == want_a


def test_infinities_saturate():
    p = np.array([-np.inf, np.inf], np.float32)
    assert q.quantize_weight(p, 0.3, 0.4).tolist() == [-1, 1]
    assert q.quantize_relu_act(p, 0.3, 0.4).tolist() == [0, 2]


def test_chain_epilogue_hand_example():
    # one pixel, four channels, numbers chosen so every float32 step is exact
    from oracle import chain
    C = np.array([[[[4, -2, 10, 1]]]], np.int32)
    scale = np.array([0.5, 0.25, 0.125, 2.0], np.float32)
    bias = np.array([-1.0, 0.0, 0.5, 0.25], np.float32)
    skip = np.array([[[[0.0, 1.0, -3.0, 0.0]]]], np.float32)
    f, lv = chain.chain_epilogue(C, scale, bias, skip, True, 1, 1.0, 1.0)
    #  f = 0.5*4-1+0 = 1 ; 0.25*-2+0+1 = 0.5 ; 0.125*10+0.5-3 = -1.25 -> relu 0 ; 2*1+0.25 = 2.25
    assert f.reshape(-1).tolist() == [1.0, 0.5, 0.0, 2.25]
    # Eq. 10 with alpha1 = alpha2 = 1: thresholds 0.5 (tie -> 0) and 1.5
    assert lv.reshape(-1).tolist() == [1, 0, 0, 2]
    f2, lv2 = chain.chain_epilogue(C, scale, bias, None, False, 0, 1.0, 1.0)
    assert f2.reshape(-1).tolist() == [1.0, -0.5, 1.75, 2.25]
    assert lv2.reshape(-1).tolist() == [2, 1, 2, 2]      # Eq. 9: -0.5 is a tie -> 0 -> level 1


def test_chain_epilogue_nan_through_relu():
    # ReLU keeps a NaN a NaN (the fp32 output shows it); the quantizer gives a NaN the value 0,
    # which is level 0 for ReLU-mode outputs and level 1 for symmetric ones
    from oracle import chain
    C = np.array([[[[4, 4]]]], np.int32)
    scale = np.array([1.0, 1.0], np.float32)
    skip = np.array([[[[np.nan, 0.0]]]], np.float32)
    for relu in (True, False):
        f, lv = chain.chain_epilogue(C, scale, None, skip, relu, 1, 1.0, 1.0)
        assert np.isnan(f.reshape(-1)[0]) and f.reshape(-1)[1] == 4.0
        assert lv.reshape(-1).tolist() == [0, 2]
        f, lv = chain.chain_epilogue(C, scale, None, skip, relu, 0, 1.0, 1.0)
        assert np.isnan(f.reshape(-1)[0]) and lv.reshape(-1).tolist() == [1, 2]
    # a negative number still goes to 0 under ReLU, and -inf too
    skip2 = np.array([[[[-10.0, -np.inf]]]], np.float32)
    f, lv = chain.chain_epilogue(C, scale, None, skip2, True, 1, 1.0, 1.0)
    assert f.reshape(-1).tolist() == [0.0, 0.0] and lv.reshape(-1).tolist() == [0, 0]


def test_quantizers_give_nan_the_value_zero_and_count_it():
    import warnings
    x = np.array([np.nan, -3.0, np.nan, 0.2, 5.0, np.inf, -np.inf], np.float32)
    with warnings.catch_warnings():
        warnings.simplefilter("error")          # no invalid-value cast, no NaN arithmetic warning
        assert q.quantize_weight(x, 0.7, 0.9).tolist() == [0, -1, 0, 0, 1, 1, -1]
        assert q.quantize_weight_piecewise(x, 0.7, 0.9).tolist() == [0, -1, 0, 0, 1, 1, -1]
        assert q.quantize_relu_act(x, 0.7, 0.9).tolist() == [0, 0, 0, 0, 2, 2, 0]
        assert q.levels_from_floats(x, True, 0, 0.7, 0.9).tolist() == [1, 0, 1, 1, 2, 2, 0]
        assert q.levels_from_floats(x, False, 1, 0.7, 0.9).tolist() == [0, 0, 0, 0, 2, 2, 0]
    assert q.count_invalid(x) == 2 and q.count_invalid(x[1:2]) == 0
