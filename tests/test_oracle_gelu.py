"""Pins for the oracle's reproducible fp32 GELU (CPU only)."""
import math

import numpy as np


def test_against_erf_gelu(vqo):
    """The tanh form is within 4.8e-4 of the erf form; allow 5e-4."""
    y = np.linspace(-8, 8, 40001).astype(np.float32)
    g = vqo.gelu(y).astype(np.float64)
    ref = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in y.astype(np.float64)])
    assert np.abs(g - ref).max() <= 5e-4
    assert np.allclose(vqo.gelu_erf(y[::1000]), ref[::1000], rtol=1e-14, atol=1e-15)


def test_against_double_tanh_form(vqo):
    """Independent evaluation with the library tanh in double: pins the constants, the cubic,
    the polynomial exponential and the 1 - 2/(1+X) rewrite to fp32 accuracy."""
    y = np.concatenate([np.linspace(-12, 12, 50001), np.linspace(-0.01, 0.01, 2001)]).astype(np.float32)
    g = vqo.gelu(y).astype(np.float64)
    yd = y.astype(np.float64)
    ref = 0.5 * yd * (1 + np.tanh(math.sqrt(2 / math.pi) * (yd + 0.044715 * yd ** 3)))
    err = np.abs(g - ref)
    assert np.all(err <= 4e-7 * np.maximum(1.0, np.abs(yd)) + 1e-9)


def test_special_values(vqo):
    g = vqo.gelu(np.array([0.0, 30.0, -30.0, 1e4, -1e4, 1.0, -1.0], np.float32))
    assert g[0] == 0.0
    assert g[1] == 30.0 and g[3] == 1e4
    assert g[2] == 0.0 and g[4] == 0.0
    assert abs(g[5] - 0.841192) < 1e-5 and abs(g[6] + 0.158808) < 1e-5


def test_minimum_of_the_dip(vqo):
    y = np.linspace(-3, 0, 30001).astype(np.float32)
    g = vqo.gelu(y)
    assert abs(float(g.min()) + 0.17004) < 2e-4
    assert abs(float(y[np.argmin(g)]) + 0.7525) < 5e-3
