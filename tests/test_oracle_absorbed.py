"""Pins for the absorbed (integer-only) linear + quantizer of the oracle: Eq. 2 in its second form
(equivalent bias inside the integer domain) with the post-scale moved into the quantizer's
references (Sec. IV-B).  The pins are exact rational arithmetic on the definition, closed forms
for power-of-two ratios, and the relation to the post-scale mode of the same oracle."""
from fractions import Fraction
import math

import numpy as np
import pytest

from oracle import vqo


def _case(seed, M, K, Nout, bits_w, bits_a):
    rng = np.random.default_rng(seed)
    lo_a, hi_a = vqo.qrange(bits_a)
    lo_w, hi_w = vqo.qrange(bits_w)
    xq = rng.integers(lo_a, hi_a + 1, size=(M, K)).astype(np.int8)
    wq = rng.integers(lo_w, hi_w + 1, size=(Nout, K)).astype(np.int8)
    s_w = (rng.uniform(0.002, 0.02, Nout)).astype(np.float32)
    bias = rng.normal(0, 0.05, Nout).astype(np.float32)
    return xq, wq, s_w, bias


def _round_half_even(fr):
    f = math.floor(fr)
    r = fr - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
        return f + 1
    return f


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_bias_and_thresholds_match_exact_rational_arithmetic(bits):
    rng = np.random.default_rng(bits)
    Nout = 24
    s_x = np.float32(0.07)
    s_w = rng.uniform(0.001, 0.03, Nout).astype(np.float32)
    bias = rng.normal(0, 0.1, Nout).astype(np.float32)
    s_y = np.float32(0.11)
    b_int, thr = vqo.absorb(s_x, s_w, bias, s_y, bits)
    lo, hi = vqo.qrange(bits)
    assert thr.shape == (Nout, hi - lo)
    for c in range(Nout):
        scale = Fraction(float(np.float32(s_x * s_w[c])))        # the fp32 product, as a rational
        assert b_int[c] == _round_half_even(Fraction(float(bias[c])) / scale)
        for t, k in enumerate(range(lo + 1, hi + 1)):
            theta = Fraction(2 * k - 1, 2) * Fraction(float(s_y)) / scale
            assert thr[c, t] == math.floor(theta), (c, k)
    assert np.all(np.diff(thr.astype(np.int64), axis=1) >= 0)


def test_power_of_two_ratio_closed_form():
    # s_y / (s_x*s_w) = 8 exactly: references (k - 1/2)*8 = 8k - 4, all integers: T = 8k - 4 and a
    # tie (a == 8k - 4) stays on the lower level
    s_x, s_w, s_y = np.float32(0.5), np.float32([0.25]), np.float32(1.0)
    b_int, thr = vqo.absorb(s_x, s_w, np.float32([3.0]), s_y, 4)
    assert b_int[0] == 24                                          # 3 / 0.125
    assert list(thr[0]) == [8 * k - 4 for k in range(-7, 8)]
    # one input row whose accumulator sweeps the references: x = a, w = 1
    for a in (-61, -60, -59, -5, -4, -3, 3, 4, 5, 51, 52, 53):
        xq = np.array([[a // 8, a - 8 * (a // 8) - 4, 4]], np.int8)     # a = 8*x0 + x1 + 4
        wq = np.array([[8, 1, 1]], np.int8)
        r = vqo.linear_absorbed(xq, wq, None, thr, 4)
        assert r["acc"][0, 0] == a
        expect = max(-8, min(7, math.ceil(Fraction(a + 4, 8)) - 1))   # number of k with a > 8k-4, from -8
        assert r["yq"][0, 0] == expect, a


@pytest.mark.parametrize("bits_w,bits_a,bits_y", [(4, 4, 4), (3, 3, 3), (2, 4, 2), (8, 8, 8)])
def test_levels_are_the_exact_comparator_decisions(bits_w, bits_a, bits_y):
    xq, wq, s_w, bias = _case(11 + bits_y, 7, 24, 9, bits_w, bits_a)
    s_x, s_y = np.float32(0.05), np.float32(0.09 if bits_y < 8 else 0.004)
    b_int, thr = vqo.absorb(s_x, s_w, bias, s_y, bits_y)
    got = vqo.linear_absorbed(xq, wq, b_int, thr, bits_y)
    assert got["overflow"] == 0
    acc = xq.astype(np.int64) @ wq.astype(np.int64).T
    assert np.array_equal(got["acc"], acc)
    lo, hi = vqo.qrange(bits_y)
    for m in range(xq.shape[0]):
        for c in range(wq.shape[0]):
            scale = Fraction(float(np.float32(s_x * s_w[c])))
            a = int(acc[m, c]) + int(b_int[c])
            # the definition in real arithmetic: references (k - 1/2)*s_y against (acc + b_int)*scale
            level = lo + sum(1 for k in range(lo + 1, hi + 1) if a * scale > Fraction(2 * k - 1, 2) * Fraction(float(s_y)))
            assert got["yq"][m, c] == level, (m, c)


def test_equivalent_bias_is_within_half_a_unit():
    rng = np.random.default_rng(3)
    s_w = rng.uniform(0.001, 0.03, 50).astype(np.float32)
    bias = rng.normal(0, 0.2, 50).astype(np.float32)
    s_x = np.float32(0.04)
    b_int, _ = vqo.absorb(s_x, s_w, bias, np.float32(0.1), 4)
    scale = (s_x * s_w).astype(np.float64)
    assert np.all(np.abs(b_int * scale - bias.astype(np.float64)) <= scale / 2 * (1 + 1e-12))
    b0, _ = vqo.absorb(s_x, s_w, None, np.float32(0.1), 4)
    assert not b0.any()


@pytest.mark.parametrize("with_bias", [False, True])
def test_relation_to_the_post_scale_mode(with_bias):
    xq, wq, s_w, bias = _case(21, 64, 96, 40, 4, 4)
    if not with_bias:
        bias = None
    s_x, s_y = np.float32(0.06), np.float32(0.05)
    post = vqo.linear(xq, s_x, wq, s_w, bias=bias, s_y=s_y, bits_y=4)
    b_int, thr = vqo.absorb(s_x, s_w, bias, s_y, 4)
    ab = vqo.linear_absorbed(xq, wq, b_int, thr, 4)
    d = ab["yq"].astype(int) - post["yq"].astype(int)
    assert np.abs(d).max() <= 1
    assert len(np.unique(post["yq"])) >= 8                      # the comparison is not vacuous
    if with_bias:
        # rounding the bias to an integer moves y by at most scale/2: only elements that close to a reference can move
        y = post["y"].astype(np.float64) / float(s_y)
        near = np.abs(y - np.floor(y) - 0.5) <= (s_x * s_w.astype(np.float64))[None, :] / float(s_y) * 0.5 + 1e-5
        assert not np.any((d != 0) & ~near)
    else:
        # without a bias the two modes see the same real number; they can only part at a tie or within fp32 rounding of it
        y = post["y"].astype(np.float64) / float(s_y)
        near = np.abs(y - np.floor(y) - 0.5) <= 1e-5
        assert not np.any((d != 0) & ~near)
        assert (d != 0).mean() < 0.01


def test_per_channel_output_steps_and_saturating_thresholds():
    s_y = np.float32([0.1, 0.2, 1e30])
    b_int, thr = vqo.absorb(np.float32(1.0), np.float32([0.01]), None, s_y, 4, Nout=3)
    assert np.all(np.abs(thr[1] - 2 * thr[0].astype(np.int64)) <= 1)      # twice the step, twice the references
    assert np.all(thr[2, :7] == -2 ** 31) and np.all(thr[2, 8:] == 2 ** 31 - 1)
    # a threshold at INT32_MAX is never exceeded, one at INT32_MIN always (except by INT32_MIN itself)
    xq = np.array([[7, 7]], np.int8)
    wq = np.array([[7, 7]] * 3, np.int8)
    r = vqo.linear_absorbed(xq, wq, None, thr, 4)
    assert r["yq"][0, 2] == -8 + 7 + (1 if 98 > thr[2, 7] else 0)
