"""Pins for the oracle's integer contractions and the reordered linear (CPU only)."""
import numpy as np
import pytest


def test_matmul_nt_vs_numpy_int64(vqo):
    rng = np.random.default_rng(5)
    for (M, N, K, bits) in ((3, 5, 7, 4), (17, 9, 130, 4), (4, 6, 64, 8), (5, 3, 33, 2)):
        lo, hi = -(2 ** (bits - 1)), 2 ** (bits - 1) - 1
        a = rng.integers(lo, hi + 1, (M, K)).astype(np.int8)
        b = rng.integers(lo, hi + 1, (N, K)).astype(np.int8)
        acc, bad = vqo.matmul_nt(a, b)
        assert bad == 0
        assert np.array_equal(acc, a.astype(np.int64) @ b.astype(np.int64).T)
        assert np.abs(acc).max() <= K * 2 ** (bits - 1) * 2 ** (bits - 1)


def test_matmul_nn_u8_vs_numpy(vqo):
    rng = np.random.default_rng(6)
    p = rng.integers(0, 256, (7, 19)).astype(np.uint8)
    v = rng.integers(-128, 128, (19, 5)).astype(np.int8)
    acc, bad = vqo.matmul_nn_u8(p, v)
    assert bad == 0
    assert np.array_equal(acc, p.astype(np.int64) @ v.astype(np.int64))


def test_extreme_operands(vqo):
    K = 3072
    a = np.full((2, K), -8, np.int8)
    assert vqo.matmul_nt(a, a)[0][0, 0] == 64 * K
    b = np.full((2, K), 7, np.int8)
    assert vqo.matmul_nt(b, a)[0][0, 0] == -56 * K
    K = 4096
    a = np.full((1, K), -128, np.int8)
    acc, bad = vqo.matmul_nt(a, a)
    assert acc[0, 0] == 2 ** 26 and bad == 0


def test_int32_overflow_is_reported(vqo):
    K = 2 ** 17                                    # (-128)^2 * 2^17 = 2^31: does not fit
    a = np.full((1, K), -128, np.int8)
    acc, bad = vqo.matmul_nt(a, a)
    assert bad == 1


def test_linear_with_unit_scales_is_integer_gemm(vqo):
    rng = np.random.default_rng(8)
    x = rng.integers(-8, 8, (6, 40)).astype(np.int8)
    w = rng.integers(-8, 8, (11, 40)).astype(np.int8)
    out = vqo.linear(x, 1.0, w, np.ones(11, np.float32))
    ref = x.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(out["acc"], ref)
    assert np.array_equal(out["y"], ref.astype(np.float32))
    assert out["overflow"] == 0


def _rand_linear(rng, M=7, K=48, N=10, bits=4):
    lo, hi = -(2 ** (bits - 1)), 2 ** (bits - 1) - 1
    x = rng.integers(lo, hi + 1, (M, K)).astype(np.int8)
    w = rng.integers(lo, hi + 1, (N, K)).astype(np.int8)
    s_w = np.exp(rng.uniform(-7, -4, N)).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    s_x = np.float32(np.exp(rng.uniform(-3, 0)))
    return x, w, s_x, s_w, b


def test_reordered_equals_dequantize_first(vqo):
    """Eq. 1 (dequantize, then multiply) and Eq. 2 (multiply, then scale) agree to fp32 rounding;
    the scaled accumulator equals the float product of the dequantized operands."""
    rng = np.random.default_rng(9)
    for bits in (2, 3, 4, 8):
        x, w, s_x, s_w, b = _rand_linear(rng, bits=bits)
        out = vqo.linear(x, s_x, w, s_w, bias=b)
        ref = vqo.linear_dequant_first(x, s_x, w, s_w, bias=b)
        # independent of the C cross-check too: numpy float64 on dequantized operands
        ref2 = (x.astype(np.float64) * float(s_x)) @ (w.astype(np.float64) * s_w[:, None].astype(np.float64)).T + b
        np.testing.assert_allclose(ref, ref2, rtol=1e-12, atol=1e-12)
        mag = np.abs(ref - b) + np.abs(b)
        assert np.all(np.abs(out["y"] - ref) <= 1e-6 * mag + 1e-9)
        nob = vqo.linear(x, s_x, w, s_w)
        ref_nob = vqo.linear_dequant_first(x, s_x, w, s_w)
        np.testing.assert_allclose(nob["y"], ref_nob, rtol=1e-6, atol=0)


def test_equivalent_bias_form_of_eq2(vqo):
    """Eq. 2's second line adds b/(s_x*s_w) inside the integer domain and scales afterwards;
    the oracle adds b after scaling.  Same value up to fp32 rounding."""
    rng = np.random.default_rng(10)
    x, w, s_x, s_w, b = _rand_linear(rng)
    out = vqo.linear(x, s_x, w, s_w, bias=b)
    acc = x.astype(np.float64) @ w.astype(np.float64).T
    sw = s_w.astype(np.float64)
    eq2 = (acc + b.astype(np.float64) / (float(s_x) * sw)) * float(s_x) * sw
    np.testing.assert_allclose(out["y"], eq2, rtol=2e-6, atol=1e-8)


def test_per_tensor_weight_step_and_no_bias(vqo):
    rng = np.random.default_rng(12)
    x, w, s_x, s_w, b = _rand_linear(rng)
    out = vqo.linear(x, s_x, w, s_w[:1])
    acc = x.astype(np.int64) @ w.astype(np.int64).T
    want = acc.astype(np.float32) * (np.float32(s_x) * s_w[0])
    assert np.array_equal(out["y"], want)


def test_requantized_output_is_quantizer_of_y(vqo):
    rng = np.random.default_rng(13)
    x, w, s_x, s_w, b = _rand_linear(rng, M=9, K=64, N=12)
    for bits_y, s_y in ((4, 0.05), (8, 0.004), (2, 0.2)):
        out = vqo.linear(x, s_x, w, s_w, bias=b, s_y=s_y, bits_y=bits_y)
        assert np.array_equal(out["yq"], vqo.quantize(out["y"], s_y, bits_y))
        assert len(np.unique(out["yq"])) > 2


def test_gelu_epilogue_applies_gelu_before_requant(vqo):
    rng = np.random.default_rng(14)
    x, w, s_x, s_w, b = _rand_linear(rng, M=5, K=64, N=8)
    s_w = s_w * 30
    plain = vqo.linear(x, s_x, w, s_w, bias=b)
    act = vqo.linear(x, s_x, w, s_w, bias=b, act=1, s_y=0.05, bits_y=4)
    assert np.array_equal(act["y"], vqo.gelu(plain["y"].ravel()).reshape(plain["y"].shape))
    assert np.array_equal(act["yq"], vqo.quantize(act["y"], 0.05, 4))
    assert np.array_equal(act["acc"], plain["acc"])
