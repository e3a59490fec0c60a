"""Pins for the oracle's uniform quantizer and weight-step rule (CPU only)."""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _thresholds():
    with open(os.path.join(GOLD, "quantizer_3bit_thresholds.txt")) as f:
        rows = [l for l in f if l.strip() and not l.startswith("#")]
    return [float(v) for v in rows[0].split()]


def test_paper_3bit_thresholds(vqo):
    """Sec. IV-B prints the 3-bit references -3.5..2.5 (x step): each separates level k-1 from k."""
    thr = _thresholds()
    assert len(thr) == 2 ** 3 - 1
    for step in (1.0, 0.25, 3.0):
        for t in thr:
            k = int(round(t + 0.5))
            eps = 2.0 ** -10
            x = np.array([[(t - eps) * step, (t + eps) * step]], np.float32)
            q = vqo.quantize(x, step, 3)
            assert q[0, 0] == k - 1 and q[0, 1] == k, (step, t, q)
    q = vqo.quantize(np.array([[-100.0, 100.0]], np.float32), 1.0, 3)
    assert q.tolist() == [[-4, 3]]


@pytest.mark.parametrize("bits", [2, 3, 4, 5, 8])
def test_level_count_and_range(vqo, bits):
    lo, hi = vqo.qrange(bits)
    assert (lo, hi) == (-(2 ** (bits - 1)), 2 ** (bits - 1) - 1)
    x = np.linspace(-300, 300, 20001, dtype=np.float32)[None, :]
    q = vqo.quantize(x, 1.0, bits)
    assert q.min() == lo and q.max() == hi
    assert len(np.unique(q)) == 2 ** bits
    assert np.all(np.diff(q[0].astype(int)) >= 0)          # monotone
    assert vqo.qrange(bits, True) == (0, 2 ** bits - 1)


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_quantize_dequantize_idempotent(vqo, bits):
    rng = np.random.default_rng(7 + bits)
    lo, hi = vqo.qrange(bits)
    levels = np.arange(lo, hi + 1, dtype=np.int8)[None, :]
    for step in np.exp(rng.uniform(-12, 6, 200)).astype(np.float32):
        x = vqo.dequantize(levels, step)
        assert np.array_equal(vqo.quantize(x, step, bits), levels)


def test_inner_thresholds_general_form(vqo):
    """(k-1/2)*step for every inner k (Sec. IV-C), 4-bit, awkward step."""
    step = np.float32(0.1)
    for k in range(-7, 8):
        t = (k - 0.5) * float(step)
        x = np.array([[t * (1 - 1e-4) if t > 0 else t * (1 + 1e-4),
                       t * (1 + 1e-4) if t > 0 else t * (1 - 1e-4)]], np.float32)
        q = vqo.quantize(x, step, 4)
        assert q[0, 0] == k - 1 and q[0, 1] == k


def test_tie_convention_is_half_to_even(vqo):
    """Convention (the paper does not fix it): exact halves go to the even level."""
    x = np.array([[0.5, 1.5, 2.5, -0.5, -1.5, -2.5]], np.float32)
    assert vqo.quantize(x, 1.0, 4).tolist() == [[0, 2, 2, 0, -2, -2]]


def test_per_row_steps_and_weight_rule(vqo):
    rng = np.random.default_rng(3)
    w = (rng.standard_normal((9, 33)) * 0.02).astype(np.float32)
    w[4] = 0.0
    for bits in (2, 3, 4, 8):
        qmax = 2 ** (bits - 1) - 1
        s = vqo.weight_steps(w, bits)
        assert s[4] == 1.0
        for r in range(9):
            if r != 4:
                # library-independent statement of the rule: absmax / qmax in fp32
                assert s[r] == np.float32(np.abs(w[r]).max()) / np.float32(qmax)
        q = vqo.quantize(w, s, bits, per_row=True)
        for r in range(9):
            if r != 4:
                assert np.abs(q[r].astype(int)).max() == qmax      # the absmax element hits +-qmax
        assert np.all(q[4] == 0)
        # each row really used its own step
        q0 = vqo.quantize(w[:1], s[0], bits)
        assert np.array_equal(q0, q[:1])


def test_matches_float32_formula_on_random(vqo):
    rng = np.random.default_rng(11)
    x = rng.standard_normal((50, 77)).astype(np.float32) * 3
    for bits, step in ((4, 0.1), (4, 0.37), (8, 0.011), (2, 1.3), (3, 0.9)):
        lo, hi = vqo.qrange(bits)
        want = np.clip(np.rint(x / np.float32(step)), lo, hi).astype(np.int8)
        assert np.array_equal(vqo.quantize(x, step, bits), want)
