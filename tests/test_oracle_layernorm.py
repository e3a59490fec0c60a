"""Pins of the oracle's LayerNorm + comparator quantizer (Sec. IV-C, Eq. 5, Fig. 5) -- CPU only.

The paper prints no worked example for this module, so the pins are: the recurrences of Eq. 5
against their closed forms (running mean, sum of squared deviations) on data where every fp32
operation is exact and against numpy in double elsewhere; the square-root-free comparator against
the direct form of Fig. 5(a) in double (agreement everywhere except within rounding distance of a
threshold); a hand-worked row; all four sign cases of the sign logic; gamma <= 0; invariances.
"""
import numpy as np
import pytest

from oracle import vqo


def _direct_levels(x, gamma, beta, eps, step, bits):
    """Fig. 5(a): y = (x-mu)/sigma*gamma+beta, level = qmin + #{k: y > (k-1/2) step}; also the margin."""
    lo, hi = vqo.qrange(bits)
    y = vqo.x_layernorm(x, gamma, beta, eps)
    ks = np.arange(lo + 1, hi + 1)
    thr = (ks - 0.5) * float(step)
    lev = lo + (y[..., None] > thr).sum(-1)
    margin = np.abs(y[..., None] - thr).min(-1)
    return lev, margin, y


def test_hand_worked_row():
    # x = (-3,-1,1,3): mean 0, sum of squared deviations 20, variance 5, sigma = 2.2360...;
    # y = (-1.3416, -0.4472, 0.4472, 1.3416); thresholds (k-1/2)/2: levels -3, -1, 1, 3
    r = vqo.layernorm_quantize(np.array([[-3, -1, 1, 3]], np.float32), np.ones(4), np.zeros(4), 0.0, 0.5, 4)
    assert r["mu"][0] == 0.0 and r["m2"][0] == 20.0
    assert r["q"].tolist() == [[-3, -1, 1, 3]]
    # beta shifts the output by one level (0.5 = one step), gamma = 2 doubles the spread
    r = vqo.layernorm_quantize(np.array([[-3, -1, 1, 3]], np.float32), np.ones(4), np.full(4, 0.5), 0.0, 0.5, 4)
    assert r["q"].tolist() == [[-2, 0, 2, 4]]
    r = vqo.layernorm_quantize(np.array([[-3, -1, 1, 3]], np.float32), np.full(4, 2.0), np.zeros(4), 0.0, 0.5, 4)
    assert r["q"].tolist() == [[-5, -2, 2, 5]]


def test_eq5_recurrences_exact_on_small_integers():
    # running means of 1..n are (i+1)/2 and the deviations' products are exact in fp32
    for n in (1, 2, 4, 8, 16, 64):
        x = np.arange(1, n + 1, dtype=np.float32)[None, :]
        r = vqo.layernorm_quantize(x, np.ones(n), np.zeros(n), 0.0, 1.0, 4)
        assert r["mu"][0] == (n + 1) / 2
        assert r["m2"][0] == n * (n * n - 1) / 12      # sum of squared deviations of 1..n


def test_eq5_recurrences_against_two_pass_double():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((50, 768)) * 3 + 1.5).astype(np.float32)
    r = vqo.layernorm_quantize(x, np.ones(768), np.zeros(768), 0.0, 0.3, 4)
    mean = x.astype(np.float64).mean(1)
    m2 = ((x.astype(np.float64) - mean[:, None]) ** 2).sum(1)
    assert np.allclose(r["mu"], mean, rtol=0, atol=2e-6)
    assert np.allclose(r["m2"], m2, rtol=2e-6)
    # it is the SUM of squared deviations, not the variance (Eq. 5 has no 1/i in its second line)
    assert np.all(r["m2"] > 100 * x.var(1))


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("eps", [0.0, 1e-5])
def test_comparator_equals_direct_form_away_from_thresholds(bits, eps):
    rng = np.random.default_rng(10 + bits)
    D = 384
    x = (rng.standard_normal((40, D)) * rng.uniform(0.2, 5, (40, 1)) + rng.uniform(-2, 2, (40, 1))).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, D).astype(np.float32)
    beta = (rng.standard_normal(D) * 0.2).astype(np.float32)
    lo, hi = vqo.qrange(bits)
    step = np.float32(3.0 / hi)
    r = vqo.layernorm_quantize(x, gamma, beta, eps, step, bits)
    lev, margin, _ = _direct_levels(x, gamma, beta, eps, step, bits)
    differ = r["q"] != lev
    assert differ.mean() < 1e-3
    assert np.all(margin[differ] < 1e-5)            # only where y sits on a threshold within fp32 rounding
    assert len(np.unique(r["q"])) >= min(hi - lo + 1, 200)   # (nearly) every level occurs: not vacuous


def test_sign_logic_all_four_cases_and_nonpositive_gamma():
    rng = np.random.default_rng(77)
    D = 64
    x = rng.standard_normal((30, D)).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, D).astype(np.float32)
    gamma[::3] *= -1                                   # negative gamma flips the data side
    gamma[5] = 0.0                                     # zero gamma: the output is quantize(beta)
    beta = rng.uniform(-1.0, 1.0, D).astype(np.float32)   # references on both sides of zero
    r = vqo.layernorm_quantize(x, gamma, beta, 1e-6, 0.25, 4)
    lev, margin, y = _direct_levels(x, gamma, beta, 1e-6, 0.25, 4)
    ok = margin > 1e-5
    assert np.array_equal(r["q"][ok], lev[ok])
    # every element is compared with all 15 references, so all four sign combinations of the
    # data side (x-mu)*gamma and the reference side (k-1/2)*step - beta are exercised
    g_pos = ((x - x.mean(1, keepdims=True)) * gamma > 0)[..., None]
    c_pos = (((np.arange(-7, 8) - 0.5) * 0.25)[None, None, :] - beta[None, :, None]) > 0
    for gs in (True, False):
        for cs in (True, False):
            assert ((g_pos == gs) & (c_pos == cs) & ok[..., None]).sum() > 1000
    assert np.all(r["q"][:, 5] == np.clip(np.rint(beta[5] / 0.25), -8, 7))


def test_invariances_and_degenerate_rows():
    rng = np.random.default_rng(3)
    D = 100
    x = rng.integers(-20, 21, (10, D)).astype(np.float32)       # small integers: shifts stay exact
    gamma = np.ones(D, np.float32)
    beta = np.zeros(D, np.float32)
    a = vqo.layernorm_quantize(x, gamma, beta, 0.0, 0.4, 4)["q"]
    # scaling the row by a power of two scales (x-mu) and sigma alike: same levels, exactly
    b = vqo.layernorm_quantize(x * 4, gamma, beta, 0.0, 0.4, 4)["q"]
    assert np.array_equal(a, b)
    # negating the data with gamma -> -gamma gives the same levels
    c = vqo.layernorm_quantize(-x, -gamma, beta, 0.0, 0.4, 4)["q"]
    assert np.array_equal(a, c)
    # a constant row: with eps > 0 the output is quantize(beta); with eps == 0 the documented qmin
    const = np.full((1, D), 3.25, np.float32)
    bq = rng.uniform(-2, 2, D).astype(np.float32)
    r = vqo.layernorm_quantize(const, gamma, bq, 1e-5, 0.4, 4)["q"]
    want = -8 + ((bq[:, None] > (np.arange(-7, 8) - 0.5) * np.float32(0.4)).sum(1))
    assert np.array_equal(r[0], want)
    assert np.all(vqo.layernorm_quantize(const, gamma, bq, 0.0, 0.4, 4)["q"] == -8)
    # normalised rows have mean beta and spread gamma (Sec. IV-C): dequantized 8-bit output
    x2 = rng.standard_normal((20, 1024)).astype(np.float32) * 7 + 3
    q = vqo.layernorm_quantize(x2, np.full(1024, 0.5), np.full(1024, 0.25), 1e-6, 0.02, 8)["q"].astype(np.float64) * 0.02
    assert np.allclose(q.mean(1), 0.25, atol=0.01) and np.allclose(q.std(1), 0.5, atol=0.01)


def test_residual_is_added_first():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((7, 48)).astype(np.float32)
    res = rng.standard_normal((7, 48)).astype(np.float32)
    g, b = np.ones(48, np.float32), np.zeros(48, np.float32)
    r = vqo.layernorm_quantize(x, g, b, 1e-6, 0.3, 4, res=res, want_sum=True)
    assert np.array_equal(r["sum"], x + res)
    assert np.array_equal(r["q"], vqo.layernorm_quantize(x + res, g, b, 1e-6, 0.3, 4)["q"])
