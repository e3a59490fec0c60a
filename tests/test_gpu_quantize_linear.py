"""GPU parity: vq_weight_steps, vq_quantize and vq_linear against the CPU oracle, bit-exact on
levels and int32 accumulators, 1e-5 rel / 1e-6 abs on fp32 (in fact expected identical)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq, workloads as wl
from tests.gpu_util import assert_fp32_close, dev, from_qmat, storage_of, to_qmat


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("shape", [(197, 384), (5, 37), (1, 1), (33, 1000)])
def test_quantize_per_tensor(bits, shape):
    rng = np.random.default_rng(100 + bits)
    x = (rng.standard_normal(shape) * 2).astype(np.float32)
    # plant exact half-way points and out-of-range values
    x.flat[: min(8, x.size)] = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 100, -100, 0], np.float32)[: min(8, x.size)] * 0.37
    step = np.float32(0.37)
    out = vitq.QMat.empty(shape[0], shape[1], bits)
    out.data.fill_(0xFF)                     # the library must overwrite the 16-byte padded row
    vitq.vq_quantize(dev(x), step, None, out)
    torch.cuda.synchronize()
    want = vqo.quantize(x, step, bits)
    assert np.array_equal(from_qmat(out), want)
    assert np.array_equal(out.data.cpu().numpy(), vqo.pack(want, storage_of(bits)))


def test_quantize_strided_input_and_per_row_steps():
    rng = np.random.default_rng(7)
    big = (rng.standard_normal((40, 100)) * 0.02).astype(np.float32)
    w = big[:, 10:77]                        # ld = 100, cols = 67, unaligned start
    big_d = dev(big)
    w_d = big_d[:, 10:77]
    for bits in (2, 3, 4, 8):
        s = vitq.vq_weight_steps(w_d, bits)
        torch.cuda.synchronize()
        s_ref = vqo.weight_steps(np.ascontiguousarray(w), bits)
        assert np.array_equal(s.cpu().numpy(), s_ref)
        out = vitq.QMat.empty(40, 67, bits)
        vitq.vq_quantize(w_d, 0.0, s, out)
        torch.cuda.synchronize()
        assert np.array_equal(from_qmat(out), vqo.quantize(np.ascontiguousarray(w), s_ref, bits, per_row=True))


def test_weight_steps_zero_row():
    w = np.zeros((3, 50), np.float32)
    w[1, 7] = -0.21
    s = vitq.vq_weight_steps(dev(w), 4).cpu().numpy()
    assert s[0] == 1.0 and s[2] == 1.0 and s[1] == np.float32(0.21) / np.float32(7)


def _run_linear(xq, s_x, wq, s_w, bias, bits_x, bits_w, act=0, s_y=None, bits_y=4, per_channel=True,
                prepack=False):
    M, Nout = xq.shape[0], wq.shape[0]
    xd, wd = to_qmat(xq, bits_x), to_qmat(wq, bits_w)
    acc = torch.full((M, Nout), -7, dtype=torch.int32, device="cuda")
    y = torch.full((M, Nout), -7.0, dtype=torch.float32, device="cuda")
    yq = vitq.QMat.empty(M, Nout, bits_y) if s_y is not None else None
    if prepack:
        wp = vitq.vq_prepack_weight(wd)
        vitq.vq_linear_prepacked(xd, s_x, wd, wp, dev(s_w), int(per_channel), dev(bias), act, acc, y,
                                 0.0 if s_y is None else s_y, yq)
    else:
        vitq.vq_linear(xd, s_x, wd, dev(s_w), int(per_channel), dev(bias), act, acc, y,
                       0.0 if s_y is None else s_y, yq)
    torch.cuda.synchronize()
    ref = vqo.linear(xq, s_x, wq, s_w, bias=bias, act=act, s_y=s_y, bits_y=bits_y)
    assert ref["overflow"] == 0
    assert np.array_equal(acc.cpu().numpy(), ref["acc"]), "int32 accumulators differ"
    assert_fp32_close(y.cpu().numpy(), ref["y"], "y")
    assert np.array_equal(y.cpu().numpy(), ref["y"]), "fp32 outputs are expected to be identical"
    if yq is not None:
        assert np.array_equal(from_qmat(yq), ref["yq"]), "requantized levels differ"
        assert np.array_equal(yq.data.cpu().numpy(), vqo.pack(ref["yq"], storage_of(bits_y)))
    return ref


def test_config1_vit_s_qkv_linear():
    """Config 1: 197x384 int4 activations (step 0.1), 1152x384 int4 weights, per-channel steps."""
    c = wl.linear_cfg1_inputs()
    xq = vqo.quantize(c["x"], c["s_x"], 4)
    s_w = vqo.weight_steps(c["w"], 4)
    wq = vqo.quantize(c["w"], s_w, 4, per_row=True)
    ref = _run_linear(xq, c["s_x"], wq, s_w, c["bias"], 4, 4)
    assert np.abs(ref["acc"]).max() > 500


def _rand_case(rng, M, K, Nout, bits_x, bits_w):
    lo_x, hi_x = vqo.qrange(bits_x)
    lo_w, hi_w = vqo.qrange(bits_w)
    xq = rng.integers(lo_x, hi_x + 1, (M, K)).astype(np.int8)
    wq = rng.integers(lo_w, hi_w + 1, (Nout, K)).astype(np.int8)
    s_w = np.exp(rng.uniform(-7, -4, Nout)).astype(np.float32)
    bias = (rng.standard_normal(Nout) * 0.01).astype(np.float32)
    return xq, wq, s_w, bias


@pytest.mark.parametrize("bits_x,bits_w", [(4, 4), (4, 3), (4, 2), (8, 8)])
@pytest.mark.parametrize("M,K,Nout", [(197, 384, 1152), (300, 100, 37), (1, 33, 1), (129, 640, 130),
                                      (64, 3072, 96)])
def test_linear_shapes_and_bit_widths(bits_x, bits_w, M, K, Nout):
    rng = np.random.default_rng(M * 7 + K + Nout + bits_w)
    xq, wq, s_w, bias = _rand_case(rng, M, K, Nout, bits_x, bits_w)
    _run_linear(xq, np.float32(0.31), wq, s_w, bias, bits_x, bits_w, s_y=np.float32(0.05), bits_y=bits_x)
    if bits_x == 4:       # the same linear through the expanded-weight kernels
        _run_linear(xq, np.float32(0.31), wq, s_w, bias, bits_x, bits_w, s_y=np.float32(0.05), bits_y=bits_x,
                    prepack=True)


@pytest.mark.parametrize("bits_x,bits_w", [(4, 4), (8, 8)])
def test_long_contraction_single_output_kernels(bits_x, bits_w):
    """K = 3072 over several token tiles with one output per call (the fp32-only and the packed-only
    epilogues; 8-bit operands take their long-contraction tile configuration): every stage of the
    software pipeline is refilled many times, and every element must be the oracle's."""
    M, K, Nout = 600, 3072, 256
    rng = np.random.default_rng(3072 + bits_w)
    xq, wq, s_w, bias = _rand_case(rng, M, K, Nout, bits_x, bits_w)
    s_x, s_y = np.float32(0.31), np.float32(0.4 if bits_x == 4 else 8.0)
    ref = vqo.linear(xq, s_x, wq, s_w, bias=bias, s_y=s_y, bits_y=bits_x)
    assert len(np.unique(ref["yq"])) >= 8
    xd, wd = to_qmat(xq, bits_x), to_qmat(wq, bits_w)
    for _ in range(3):
        y = torch.full((M, Nout), -7.0, dtype=torch.float32, device="cuda")
        vitq.vq_linear(xd, s_x, wd, dev(s_w), 1, dev(bias), 0, None, y, 0.0, None)
        yq = vitq.QMat.empty(M, Nout, bits_x)
        vitq.vq_linear(xd, s_x, wd, dev(s_w), 1, dev(bias), 0, None, None, s_y, yq)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), ref["y"])
        assert np.array_equal(from_qmat(yq), ref["yq"])


def test_fast_gelu_stays_within_the_bound_its_guard_assumes():
    """The GELU + requantizing epilogue accepts a level from the hardware exp2 / rcp form of the activation
    only when it is further than 2^-21 * |y| / s_y from a rounding boundary.  That is sound as long as the
    fast form is within 2^-21 * |y| of the definition's for EVERY fp32 y: run through all of them."""
    worst = vitq.vq_probe_gelu_distance()
    torch.cuda.synchronize()
    assert 0.0 < float(worst.item()) <= 2.0 ** -22, "fast GELU drifts %g * |y| from the definition" % worst.item()


@pytest.mark.parametrize("s_y", [0.0028, 0.047, 0.35])
def test_gelu_requant_only_output_matches_the_definition_on_dense_inputs(s_y):
    """Packed-only output with GELU (the guarded epilogue), on y values swept densely through the range in
    which the sixteen levels change: with zero weights y is the bias, one value per channel."""
    M, K, Nout = 64, 64, 4096
    lo, hi = vqo.qrange(4)
    y_span = (hi + 1.5) * s_y + 0.2
    bias = np.linspace(-min(4.0, 12 * y_span), y_span, Nout).astype(np.float32)
    rng = np.random.default_rng(5)
    bias += (rng.standard_normal(Nout) * 1e-4).astype(np.float32)
    # ... and the fp32 neighbourhoods (+-32 ulps) of the points where the definition's level changes on the
    # rising branch: both sides of every guard band
    near = []
    for k in range(lo + 1, hi + 1):
        target = (k - 0.5) * float(s_y)
        a_, b_ = -0.75, 20.0
        if not (float(vqo.gelu(np.float32(a_))[0]) < target < float(vqo.gelu(np.float32(b_))[0])):
            continue
        for _ in range(60):
            m_ = 0.5 * (a_ + b_)
            if float(vqo.gelu(np.float32(m_))[0]) < target:
                a_ = m_
            else:
                b_ = m_
        y0 = np.float32(b_)
        up, dn = y0, y0
        near.append(y0)
        for _ in range(32):
            up = np.nextafter(up, np.float32(np.inf), dtype=np.float32)
            dn = np.nextafter(dn, np.float32(-np.inf), dtype=np.float32)
            near += [up, dn]
    near = np.array(near, np.float32)
    assert near.size >= 65 * 7
    bias[:near.size] = near
    xq = rng.integers(lo, hi + 1, (M, K)).astype(np.int8)
    wq = np.zeros((Nout, K), np.int8)
    s_w = np.ones(Nout, np.float32)
    ref = vqo.linear(xq, np.float32(0.5), wq, s_w, bias=bias, act=1, s_y=np.float32(s_y), bits_y=4)
    assert len(np.unique(ref["yq"])) >= 8
    yq = vitq.QMat.empty(M, Nout, 4)
    vitq.vq_linear(to_qmat(xq, 4), np.float32(0.5), to_qmat(wq, 4), dev(s_w), 1, dev(bias), 1, None, None,
                   np.float32(s_y), yq)
    torch.cuda.synchronize()
    got = from_qmat(yq)
    assert np.array_equal(got, ref["yq"]), "levels differ at y = %r" % bias[np.flatnonzero((got != ref["yq"]).any(0))[:8]]


def test_prepacked_weights_are_the_levels_in_operand_order():
    rng = np.random.default_rng(91)
    perm = [0, 2, 4, 6, 1, 3, 5, 7, 8, 10, 12, 14, 9, 11, 13, 15]
    for bits, cols in ((4, 100), (3, 33), (2, 64), (4, 16)):
        lo, hi = vqo.qrange(bits)
        wq = rng.integers(lo, hi + 1, (37, cols)).astype(np.int8)
        wp = vitq.vq_prepack_weight(to_qmat(wq, bits)).cpu().numpy().view(np.int8)
        kp = (cols + 15) // 16 * 16
        want = np.zeros((37, kp), np.int8)
        want[:, :cols] = wq
        want = want.reshape(37, kp // 16, 16)[:, :, perm].reshape(37, kp)
        assert np.array_equal(wp[: 37 * kp].reshape(37, kp), want)


@pytest.mark.parametrize("bits_x,bits_w", [(4, 4), (4, 2), (8, 8)])
def test_linear_extreme_operands(bits_x, bits_w):
    lo_x, hi_x = vqo.qrange(bits_x)
    lo_w, hi_w = vqo.qrange(bits_w)
    K = 4096
    for xv, wv in ((lo_x, lo_w), (hi_x, lo_w), (lo_x, hi_w)):
        xq = np.full((40, K), xv, np.int8)
        wq = np.full((70, K), wv, np.int8)
        ref = _run_linear(xq, np.float32(1.0), wq, np.ones(70, np.float32), None, bits_x, bits_w)
        assert ref["acc"][0, 0] == xv * wv * K
        if bits_x == 4:
            _run_linear(xq, np.float32(1.0), wq, np.ones(70, np.float32), None, bits_x, bits_w, prepack=True)


def test_linear_gelu_requant_and_per_tensor_weight_step():
    rng = np.random.default_rng(55)
    xq, wq, s_w, bias = _rand_case(rng, 150, 256, 200, 4, 4)
    s_w = (s_w * 40).astype(np.float32)
    ref = _run_linear(xq, np.float32(0.2), wq, s_w, bias, 4, 4, act=1, s_y=np.float32(0.12), bits_y=4)
    assert len(np.unique(ref["yq"])) >= 8
    _run_linear(xq, np.float32(0.2), wq, s_w[:1], None, 4, 4, per_channel=False)
    _run_linear(xq, np.float32(0.2), wq, s_w, bias, 4, 4, act=1, s_y=np.float32(0.004), bits_y=8)
    _run_linear(xq, np.float32(0.2), wq, s_w, bias, 4, 4, s_y=np.float32(0.5), bits_y=2)
    _run_linear(xq, np.float32(0.2), wq, s_w, bias, 4, 4, act=1, s_y=np.float32(0.12), bits_y=4, prepack=True)
    _run_linear(xq, np.float32(0.2), wq, s_w, bias, 4, 4, act=1, s_y=np.float32(0.004), bits_y=8, prepack=True)


@pytest.mark.parametrize("bits_y", [2, 3, 4, 5, 7, 8])
def test_linear_requant_to_every_level_count(bits_y):
    """Levels narrower than their storage field (3 bits in a nibble, 5..7 in a byte) take the same epilogues."""
    rng = np.random.default_rng(300 + bits_y)
    xq, wq, s_w, bias = _rand_case(rng, 130, 192, 160, 4, 4)
    s_w = (s_w * 40).astype(np.float32)
    s_y = np.float32(1.2 / (1 << (bits_y - 1)))
    for act in (0, 1):
        ref = _run_linear(xq, np.float32(0.2), wq, s_w, bias, 4, 4, act=act, s_y=s_y, bits_y=bits_y)
        lo, hi = vqo.qrange(bits_y)
        assert ref["yq"].min() == lo or act == 1
        assert ref["yq"].max() == hi


def test_linear_only_requested_outputs_are_written_and_runs_are_deterministic():
    rng = np.random.default_rng(56)
    xq, wq, s_w, bias = _rand_case(rng, 197, 384, 384, 4, 4)
    xd, wd = to_qmat(xq, 4), to_qmat(wq, 4)
    outs = []
    for _ in range(2):
        yq = vitq.QMat.empty(197, 384, 4)
        vitq.vq_linear(xd, 0.3, wd, dev(s_w), 1, dev(bias), 0, None, None, 0.07, yq)
        torch.cuda.synchronize()
        outs.append(yq.data.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])
    ref = vqo.linear(xq, np.float32(0.3), wq, s_w, bias=bias, s_y=np.float32(0.07), bits_y=4)
    assert np.array_equal(outs[0], vqo.pack(ref["yq"], 4))


def test_failed_check_leaves_outputs_untouched():
    rng = np.random.default_rng(57)
    xq, wq, s_w, bias = _rand_case(rng, 10, 64, 16, 4, 4)
    xd, wd = to_qmat(xq, 4), to_qmat(wq, 4)
    y = torch.full((10, 16), 3.0, device="cuda")
    with pytest.raises(vitq.VitqError) as e:
        vitq.vq_linear(xd, float("inf"), wd, dev(s_w), 1, None, 0, None, y, 0.0, None)
    assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_STEP")
    torch.cuda.synchronize()
    assert torch.all(y == 3.0)


@pytest.mark.parametrize("bits,Nout", [(4, 48), (8, 16), (3, 80)])
def test_requantized_only_output_keeps_the_row_padding_zero(bits, Nout):
    # only yq requested: the specialised epilogue runs; the bytes between the last channel and the
    # 16-byte padded row end must come out zero (the next linear reads them as operand values)
    rng = np.random.default_rng(bits + Nout)
    xq, wq, s_w, bias = _rand_case(rng, 70, 128, Nout, bits, bits)
    xd, wd = to_qmat(xq, bits), to_qmat(wq, bits)
    yq = vitq.QMat.empty(70, Nout, bits)
    yq.data.fill_(0xEE)
    vitq.vq_linear(xd, np.float32(0.31), wd, dev(s_w), 1, dev(bias), 0, None, None, np.float32(0.05), yq)
    torch.cuda.synchronize()
    ref = vqo.linear(xq, np.float32(0.31), wq, s_w, bias=bias, s_y=np.float32(0.05), bits_y=bits)
    assert np.array_equal(yq.data.cpu().numpy(), vqo.pack(ref["yq"], storage_of(bits)))
