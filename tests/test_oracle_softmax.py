"""Pins for the shift-based exponential and the row-sum-scaled softmax quantizer (CPU only)."""
import math

import numpy as np
import pytest

ONE = 1 << 20


def test_alpha_is_three_multiplies_times_log2e(vqo):
    a = vqo.alpha(0.3, 0.7, 0.125)
    want = np.float32(np.float32(np.float32(np.float32(0.3) * np.float32(0.7)) * np.float32(0.125))
                      * np.float32(1.44269504))
    assert a == want
    assert abs(float(a) - 0.3 * 0.7 * 0.125 * math.log2(math.e)) < 1e-7


def test_shift_exp_powers_of_two_when_exponent_is_integer(vqo):
    """Eq. 4 with r = 0: the exponential is a pure shift."""
    for d in range(0, -40, -1):
        e = vqo.shift_exp(d, 1.0)
        assert e == (ONE >> min(-d, 31)), d
    assert vqo.shift_exp(-64, 0.5) == ONE >> 31 == 0
    assert vqo.shift_exp(-4, 0.5) == ONE >> 2


def test_shift_exp_linearised_fraction(vqo):
    """Eq. 4: 2^(f+r) ~ (1+r) << f.  alpha = 1/4 makes r one of 0, .25, .5, .75 exactly."""
    for d in range(0, -60, -1):
        t = 0.25 * d
        f = math.floor(t)
        r = t - f
        want = int((1.0 + r) * ONE) >> min(-f, 31)
        assert vqo.shift_exp(d, 0.25) == want


def test_shift_exp_error_band(vqo):
    """(1+r)/2^r lies in [1, 1.0615] (maximum at r = 1/ln2 - 1), so the fixed-point value stays
    within that band of the true 2^(alpha*d), up to the truncation of the shift."""
    rng = np.random.default_rng(2)
    for alpha in (0.013, 0.11, 0.9, 2.3):
        for d in rng.integers(-int(18 / alpha), 1, 300):
            e = vqo.shift_exp(int(d), alpha)
            t = float(np.float32(alpha) * np.float32(d))
            true = ONE * 2.0 ** t
            assert e <= true * 1.0616 + 1
            assert e >= true * 0.99999 - 1.0       # truncation loses < 1 unit


def test_one_hot_and_uniform_rows(vqo):
    s = np.full(197, -4000, np.int32)
    s[17] = 3000
    p, e, tot = vqo.softmax_row(s, 0.05, 15)
    assert p[17] == 15 and p.sum() == 15 and tot == ONE
    # uniform row: every term is 2^20, level = round(pmax / N)
    for n, pmax, want in ((197, 15, 0), (577, 15, 0), (7, 15, 2), (4, 15, 4), (9, 15, 2),
                         (10, 15, 1), (2, 255, 127)):  # 15/10 and 255/2: exact ties, down
        p, e, tot = vqo.softmax_row(np.full(n, 123, np.int32), 0.3, pmax)
        assert tot == n * ONE and np.all(e == ONE)
        assert np.all(p == want), (n, pmax, p[:4])


def test_exact_tie_goes_down(vqo):
    """Two equal maxima, everything else negligible: the ratio is pmax/2 = 7.5 at 4 bits, an
    exact tie of the strict comparator (reading: tie -> lower level)."""
    s = np.full(50, -100000, np.int32)
    s[3] = s[40] = 77
    p, e, tot = vqo.softmax_row(s, 1.0, 15)
    assert tot == 2 * ONE
    assert p[3] == 7 and p[40] == 7 and p.sum() == 14
    p, _, _ = vqo.softmax_row(s, 1.0, 255)
    assert p[3] == 127 and p[40] == 127                  # 127.5 ties down too


def test_closed_form_when_terms_are_exact_powers_of_two(vqo):
    """With alpha*d integer the quantizer input is an exact base-2 softmax; compare with exact
    rational arithmetic: level = #{k : 2*pmax*e > (2k-1)*sum}."""
    from fractions import Fraction
    rng = np.random.default_rng(4)
    for _ in range(30):
        n = int(rng.integers(2, 40))
        s = rng.integers(-12, 1, n).astype(np.int32)
        s[rng.integers(0, n)] = 0
        p, e, tot = vqo.softmax_row(s, 1.0, 15)
        w = [Fraction(1, 2 ** int(-v)) for v in s]
        z = sum(w)
        for j in range(n):
            ratio = 15 * w[j] / z                       # pmax * softmax_j, exact
            want = sum(1 for k in range(1, 16) if ratio > Fraction(2 * k - 1, 2))
            assert p[j] == want


def test_counting_form_equals_division_form(vqo):
    rng = np.random.default_rng(5)
    for pmax in (15, 255, 7):
        s = rng.integers(-300, 300, 197).astype(np.int32)
        p, e, tot = vqo.softmax_row(s, 0.021, pmax)
        e64 = e.astype(np.int64)
        closed = np.minimum(pmax, (2 * pmax * e64 + tot - 1) // (2 * tot))
        assert np.array_equal(p.astype(np.int64), closed)
        assert tot == int(e64.sum())
        assert e.max() == ONE


def test_within_one_level_of_true_softmax(vqo):
    rng = np.random.default_rng(6)
    worst = 0
    for trial in range(40):
        n = int(rng.choice([37, 197, 198, 577]))
        s_q, s_k = np.float32(rng.uniform(0.05, 0.6)), np.float32(rng.uniform(0.05, 0.6))
        s = np.rint(rng.standard_normal(n) * rng.uniform(5, 400)).astype(np.int32)
        a = vqo.alpha(s_q, s_k, 0.125)
        for pmax in (15, 255):
            p, e, tot = vqo.softmax_row(s, a, pmax)
            pt, prob = vqo.softmax_true(s, float(s_q) * float(s_k) * 0.125, pmax)
            # the linearised exponential is off by at most 6.15 % per term, so the normalised
            # value moves by at most that factor either way
            lo = np.floor(prob * pmax / 1.0616 + 0.5 - 1e-9)
            hi = np.ceil(prob * pmax * 1.0616 + 0.5 + 1e-9)
            assert np.all(p >= lo - 1e-9) and np.all(p <= hi)
            if pmax == 15:
                worst = max(worst, int(np.abs(p.astype(int) - pt.astype(int)).max()))
                assert np.abs(p.astype(int) - pt.astype(int)).max() <= 1
            assert pmax - n / 2 <= int(p.sum()) <= pmax + n / 2


def test_shift_invariance_and_argmax(vqo):
    rng = np.random.default_rng(7)
    s = rng.integers(-500, 500, 197).astype(np.int32)
    a = vqo.alpha(0.31, 0.27, 0.125)
    p0, _, _ = vqo.softmax_row(s, a, 15)
    for c in (-4096, 1, 100000):
        p1, _, _ = vqo.softmax_row(s + np.int32(c), a, 15)
        assert np.array_equal(p0, p1)
    assert p0[np.argmax(s)] == p0.max()
    order = np.argsort(s)
    assert np.all(np.diff(p0[order].astype(int)) >= 0)      # monotone in the score


def test_single_element_row(vqo):
    p, e, tot = vqo.softmax_row(np.array([5], np.int32), 0.1, 15)
    assert p[0] == 15 and tot == ONE
