"""GPU parity: vq_layernorm_quantize against the CPU oracle -- levels and packed bytes bit-exact
(both sides run Eq. 5 in fp32 in element order and decide with the same comparator arithmetic),
the residual sum identical."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq
from tests.gpu_util import dev, from_qmat, storage_of


def _case(rng, rows, cols, scale=1.0):
    x = (rng.standard_normal((rows, cols)) * rng.uniform(0.2, 4.0, (rows, 1)) * scale
         + rng.uniform(-2, 2, (rows, 1))).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, cols).astype(np.float32)
    beta = (rng.standard_normal(cols) * 0.3).astype(np.float32)
    return x, gamma, beta


def _check(x, gamma, beta, eps, step, bits, res=None, ld=None):
    rows, cols = x.shape
    out = vitq.QMat.empty(rows, cols, bits)
    out.data.fill_(0xFF)                      # the whole 16-byte padded row must be overwritten
    if ld is None:
        xd, rd = dev(x), dev(res)
    else:                                     # rows embedded in a wider buffer
        big = torch.zeros((rows, ld), dtype=torch.float32, device="cuda")
        big[:, :cols] = dev(x)
        xd = big[:, :cols]
        rd = None
        if res is not None:
            bigr = torch.zeros((rows, ld), dtype=torch.float32, device="cuda")
            bigr[:, :cols] = dev(res)
            rd = bigr[:, :cols]
    sd = torch.full((rows, ld or cols), -7.0, dtype=torch.float32, device="cuda")[:, :cols] if res is not None else None
    vitq.vq_layernorm_quantize(xd, rd, sd, dev(gamma), dev(beta), eps, step, out)
    torch.cuda.synchronize()
    ref = vqo.layernorm_quantize(x, gamma, beta, eps, step, bits, res=res, want_sum=res is not None)
    got = from_qmat(out)
    assert np.array_equal(got, ref["q"]), "levels differ: %d of %d" % ((got != ref["q"]).sum(), got.size)
    assert np.array_equal(out.data.cpu().numpy(), vqo.pack(ref["q"], storage_of(bits)))
    if res is not None:
        assert np.array_equal(sd.cpu().numpy(), ref["sum"])
    return ref


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("rows,cols", [(197, 384), (130, 768), (3, 1024), (70, 37), (1, 1), (65, 5), (64, 130)])
def test_shapes_and_bit_widths(bits, rows, cols):
    rng = np.random.default_rng(rows * 31 + cols + bits)
    x, gamma, beta = _case(rng, rows, cols)
    lo, hi = vqo.qrange(bits)
    ref = _check(x, gamma, beta, 1e-5, np.float32(2.5 / hi), bits)
    if rows * cols > 5000:
        assert len(np.unique(ref["q"])) >= min(hi - lo + 1, 100)


def test_residual_strided_rows_and_no_eps():
    rng = np.random.default_rng(9)
    x, gamma, beta = _case(rng, 100, 384)
    res = rng.standard_normal((100, 384)).astype(np.float32)
    _check(x, gamma, beta, 0.0, np.float32(0.35), 4, res=res)
    _check(x, gamma, beta, 1e-6, np.float32(0.35), 4, res=res, ld=400)
    _check(x[:, :383], gamma[:383], beta[:383], 1e-6, np.float32(0.35), 4, res=res[:, :383], ld=400)   # unaligned


def test_gamma_of_any_sign_constant_rows_and_extreme_values():
    rng = np.random.default_rng(10)
    x, gamma, beta = _case(rng, 80, 256)
    gamma[::3] *= -1
    gamma[7] = 0.0
    x[3, :] = 1.75                            # constant row
    x[4, :] = 0.0
    x[5, :] *= 1e18                           # squares overflow to inf on both sides alike
    x[6, :] *= 1e-20                          # squares underflow
    x[8, 17] = np.inf
    x[9, 0] = np.nan                          # every comparison false from there on
    # deviations outside the range in which the kernel replaces the division of Eq. 5 by a corrected
    # reciprocal multiply (it must notice and divide), and one row that mixes both regimes
    x[10, :] *= 1e37
    x[11, :] *= 1e-33
    x[12, :] *= 1e-41                         # subnormal inputs
    x[13, 40:] *= 1e-36
    x[14, :] = 3.0e-38
    x[14, 100] = 3.0000004e-38                # a subnormal deviation from an ordinary mean
    for eps in (0.0, 1e-5):
        _check(x, gamma, beta, eps, np.float32(0.3), 4)
    _check(x, gamma, beta, 1e-5, np.float32(0.02), 8)


def test_block_sized_input_sampled():
    """The benchmark's size (50,432 x 768): the whole matrix on the GPU, sampled rows by the oracle."""
    rng = np.random.default_rng(11)
    rows, cols = 256 * 197, 768
    x = torch.randn((rows, cols), generator=torch.Generator().manual_seed(5)).numpy()
    gamma = rng.uniform(0.5, 1.5, cols).astype(np.float32)
    beta = (rng.standard_normal(cols) * 0.3).astype(np.float32)
    out = vitq.QMat.empty(rows, cols, 4)
    vitq.vq_layernorm_quantize(dev(x), None, None, dev(gamma), dev(beta), 1e-5, 0.4, out)
    torch.cuda.synchronize()
    sample = np.r_[0:64, 25000:25064, rows - 64:rows]
    ref = vqo.layernorm_quantize(x[sample], gamma, beta, 1e-5, 0.4, 4)
    got = vqo.unpack(out.data.cpu().numpy()[sample], cols, 4)
    assert np.array_equal(got, ref["q"])


def test_bad_arguments_leave_output_untouched():
    out = vitq.QMat.empty(4, 8, 4)
    out.data.fill_(0x5A)
    x = torch.zeros((4, 8), device="cuda")
    g = torch.ones(8, device="cuda")
    for eps, step in ((-1.0, 0.5), (0.0, 0.0), (float("nan"), 0.5)):
        with pytest.raises(vitq.VitqError) as e:
            vitq.vq_layernorm_quantize(x, None, None, g, g, eps, step, out)
        assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_STEP")
    torch.cuda.synchronize()
    assert torch.all(out.data == 0x5A)


def test_every_binary_exponent_of_the_input_scale():
    # one row per power of two from 2^-140 to 2^126: the kernel's division-free mean update is only
    # used while the deviations are ordinary numbers, and must hand over to the division outside
    # that range without a visible seam (both sides overflow and underflow alike)
    rng = np.random.default_rng(77)
    exps = np.arange(-140, 127)
    cols = 200
    base = rng.standard_normal((len(exps), cols)).astype(np.float32)
    with np.errstate(over="ignore", under="ignore"):
        x = (base.astype(np.float64) * np.exp2(exps.astype(np.float64))[:, None]).astype(np.float32)
    x[5, 10:60] = 0.0                          # exact zero deviations inside a tiny row
    x[200, 3] = x[200, 4]                      # a repeated value
    gamma = rng.uniform(0.5, 1.5, cols).astype(np.float32)
    beta = rng.normal(0, 0.3, cols).astype(np.float32)
    for eps in (0.0, 1e-6):
        _check(x, gamma, beta, eps, np.float32(0.4), 4)


@pytest.mark.parametrize("bits,gsign", [(4, 1.0), (4, -1.0), (8, 1.0), (3, 1.0)])
def test_values_planted_on_both_sides_of_every_guard_band(bits, gsign):
    """A guessed level stands without the comparator when it is provably far from a boundary.  beta is chosen
    per column so that one element of that column sits a chosen distance (2^-27 .. 2^-12 levels, either
    side) from a comparator boundary; every level must still be the oracle's."""
    rows, cols, eps = 64, 768, np.float32(1e-6)
    rng = np.random.default_rng(900 + bits)
    x, gamma, _ = _case(rng, rows, cols)
    gamma = (gamma * gsign).astype(np.float32)
    lo, hi = vqo.qrange(bits)
    step = np.float32(4.0 / hi)
    # Eq. 5 in fp32, element order, all rows at once (the statistics do not depend on beta)
    mu = np.zeros(rows, np.float32)
    m2 = np.zeros(rows, np.float32)
    for i in range(cols):
        d1 = x[:, i] - mu
        mu = mu + d1 / np.float32(i + 1)
        m2 = m2 + d1 * (x[:, i] - mu)
    V = (m2 + np.float32(cols) * eps).astype(np.float64)
    sigma = np.sqrt(V / cols)
    beta = np.zeros(cols, np.float32)
    for j in range(cols):
        r = j % rows
        g = np.float32(np.float32(x[r, j] - mu[r]) * gamma[j])
        k = int(rng.integers(lo + 1, hi + 1))
        delta = float(rng.choice([-1.0, 1.0])) * 2.0 ** float(rng.uniform(-27, -12))
        beta[j] = np.float32(float(step) * (k - 0.5 + delta) - float(g) / sigma[r])
    _check(x, gamma, beta, eps, step, bits)
