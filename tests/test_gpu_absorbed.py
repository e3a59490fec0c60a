"""GPU parity: vq_linear_absorbed (integer-only linear + quantizer: equivalent bias in the integer
domain, scales absorbed into the comparator references) against the CPU oracle, bit-exact."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq
from tests.gpu_util import dev, from_qmat, to_qmat


def _operands(seed, M, K, Nout, bits_w, bits_a):
    rng = np.random.default_rng(seed)
    lo_a, hi_a = vqo.qrange(bits_a)
    lo_w, hi_w = vqo.qrange(bits_w)
    xq = rng.integers(lo_a, hi_a + 1, size=(M, K)).astype(np.int8)
    wq = rng.integers(lo_w, hi_w + 1, size=(Nout, K)).astype(np.int8)
    s_w = rng.uniform(0.002, 0.02, Nout).astype(np.float32)
    bias = rng.normal(0, 0.05, Nout).astype(np.float32)
    return xq, wq, s_w, bias


def _run(xq, wq, b_int, thr, bits_w, bits_a, bits_y, want_acc=True, sum_may_leave_int32=False):
    M, Nout = xq.shape[0], wq.shape[0]
    xd, wd = to_qmat(xq, bits_a), to_qmat(wq, bits_w)
    out = vitq.QMat.empty(M, Nout, bits_y, storage_bits=4 if bits_y <= 4 else 8)   # 2-bit levels in 4-bit fields
    out.data.fill_(0xFF)
    acc = torch.full((M, Nout), -7, dtype=torch.int32, device="cuda") if want_acc else None
    bd = None if b_int is None else torch.from_numpy(np.ascontiguousarray(b_int)).cuda()
    td = torch.from_numpy(np.ascontiguousarray(thr)).cuda()
    vitq.vq_linear_absorbed(xd, wd, bd, td, acc, out)
    torch.cuda.synchronize()
    ref = vqo.linear_absorbed(xq, wq, b_int, thr, bits_y)
    assert sum_may_leave_int32 or ref["overflow"] == 0
    got = from_qmat(out)
    assert np.array_equal(got, ref["yq"]), "levels differ at %d of %d" % ((got != ref["yq"]).sum(), got.size)
    assert np.array_equal(out.data.cpu().numpy(), vqo.pack(ref["yq"], out.storage_bits))
    if want_acc:
        assert np.array_equal(acc.cpu().numpy(), ref["acc"])
    return ref


@pytest.mark.parametrize("bits_w,bits_a,bits_y,M,K,Nout", [
    (4, 4, 4, 300, 200, 48),        # ragged token tile, K tail, one partial channel tile
    (4, 4, 4, 591, 768, 768),       # the projection of three ViT-B images
    (4, 4, 3, 130, 384, 144),
    (4, 4, 2, 64, 96, 16),
    (3, 3, 3, 197, 384, 384),
    (2, 4, 4, 77, 160, 32),
    (8, 8, 8, 150, 320, 64),        # 255 references per channel: read from global memory
    (8, 8, 4, 129, 64, 160),
    (4, 4, 8, 40, 128, 32),
    (8, 8, 6, 70, 128, 32),         # 63 references: both levels of the two-level table end early
    (4, 4, 5, 33, 256, 48),         # 31 references
    (8, 8, 7, 20, 64, 16),          # 127 references
])
def test_against_oracle(bits_w, bits_a, bits_y, M, K, Nout):
    xq, wq, s_w, bias = _operands(1000 + M + bits_y, M, K, Nout, bits_w, bits_a)
    s_x = np.float32(0.05)
    acc_std = float(np.std(xq.astype(np.int64) @ wq.astype(np.int64).T * (s_x * s_w)[None, :]))
    lo, hi = vqo.qrange(bits_y)
    s_y = np.float32(2.5 * acc_std / hi)                           # levels spread over the whole range
    b_int, thr = vitq.vq_absorb_thresholds(s_x, s_w, bias, [s_y], bits_y)
    b_ref, thr_ref = vqo.absorb(s_x, s_w, bias, s_y, bits_y)
    assert np.array_equal(b_int, b_ref) and np.array_equal(thr, thr_ref)
    ref = _run(xq, wq, b_int, thr, bits_w, bits_a, bits_y)
    assert len(np.unique(ref["yq"])) >= min(hi - lo + 1, 12) - 2


def test_no_bias_and_per_channel_output_steps():
    xq, wq, s_w, _ = _operands(5, 100, 256, 96, 4, 4)
    s_y = np.random.default_rng(6).uniform(0.02, 0.4, 96).astype(np.float32)
    b_int, thr = vitq.vq_absorb_thresholds(0.05, s_w, None, s_y, 4)
    assert not b_int.any()
    _run(xq, wq, None, thr, 4, 4, 4, want_acc=False)


def test_irregular_reference_tables():
    # references that are far from equally spaced, repeated, or saturated: the count must still be exact
    xq, wq, _, _ = _operands(9, 200, 128, 32, 4, 4)
    rng = np.random.default_rng(10)
    thr = np.sort(rng.integers(-900, 900, size=(32, 15)), axis=1).astype(np.int32)
    thr[0, :] = 17                                   # all equal
    thr[1, :5] = -2 ** 31
    thr[1, 5:] = 2 ** 31 - 1                         # five always exceeded (but by INT32_MIN), ten never
    thr[2, :] = np.sort(np.r_[rng.integers(-5, 5, 14), 100000]).astype(np.int32)   # one far outlier
    thr[3, :] = np.arange(15) - 7                    # unit spacing around zero
    thr[4, 7:] = thr[4, 7]                           # upper half collapsed
    b_int = rng.integers(-50, 50, 32).astype(np.int32)
    ref = _run(xq, wq, b_int, thr, 4, 4, 4)
    assert set(np.unique(ref["yq"][:, 0])) <= {-8, 7}
    assert np.all(ref["yq"][:, 1] == -3)


def test_equivalent_bias_at_the_int32_limits():
    """b_int is clamped to int32 by the preparation step, so a near-dead channel carries INT32_MAX or
    INT32_MIN; the sum with an accumulator of the same sign then leaves 32 bits, and the oracle
    compares it in 64 bits.  Accumulators of both signs, references at and next to the limits."""
    xq, wq, _, _ = _operands(21, 160, 192, 48, 4, 4)
    rng = np.random.default_rng(22)
    thr = np.sort(rng.integers(-3000, 3000, size=(48, 15)), axis=1).astype(np.int32)
    b_int = rng.integers(-50, 50, 48).astype(np.int32)
    imax, imin = 2 ** 31 - 1, -2 ** 31
    b_int[0], thr[0, :] = imax, imax                     # exceeded only by sums above INT32_MAX
    b_int[1], thr[1, :] = imin, imin                     # exceeded unless the sum is INT32_MIN or below
    b_int[2], thr[2, :] = imax, np.sort(np.r_[np.full(8, imax - 1), np.full(7, imax)])
    b_int[3], thr[3, :] = imin, np.sort(np.r_[np.full(5, imin), np.full(10, imin + 40)])
    b_int[4], thr[4, :] = imax - 1000, imax - np.arange(15)[::-1] * 150
    b_int[5], thr[5, :] = imin + 1000, imin + np.arange(15) * 150
    b_int[17], thr[17, :] = imax, np.sort(rng.integers(-3000, 3000, 15))   # ordinary references, huge bias
    b_int[33], thr[33, :] = imin, np.sort(rng.integers(-3000, 3000, 15))
    ref = _run(xq, wq, b_int, thr, 4, 4, 4, sum_may_leave_int32=True)
    acc = ref["acc"]
    assert (acc[:, 0] > 0).any() and (acc[:, 0] < 0).any()                 # both signs meet the limits
    assert len(np.unique(ref["yq"][:, 0])) == 2 and len(np.unique(ref["yq"][:, 1])) == 2
    assert np.all(ref["yq"][:, 17] == 7) and np.all(ref["yq"][:, 33] == -8)
    # the same through the two-level table of more than fifteen references per channel
    thr8 = np.sort(rng.integers(-3000, 3000, size=(48, 255)), axis=1).astype(np.int32)
    thr8[0, :], thr8[1, :] = imax, imin
    thr8[2, :128], thr8[2, 128:] = imax - 1, imax
    _run(xq, wq, b_int, thr8, 4, 4, 8, sum_may_leave_int32=True)


def test_argument_errors():
    xq, wq, s_w, bias = _operands(3, 8, 64, 24, 4, 4)       # 24 output channels: not a multiple of 16
    b_int, thr = vitq.vq_absorb_thresholds(0.05, s_w, bias, [0.1], 4)
    xd, wd = to_qmat(xq, 4), to_qmat(wq, 4)
    out = vitq.QMat.empty(8, 24, 4)
    td = torch.from_numpy(thr).cuda()
    with pytest.raises(vitq.VitqError) as e:
        vitq.vq_linear_absorbed(xd, wd, None, td, None, out)
    assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_UNSUPPORTED")
    with pytest.raises(vitq.VitqError) as e:
        vitq.vq_linear_absorbed(xd, wd, None, None, None, out)
    assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_NULL")
    with pytest.raises(vitq.VitqError) as e:
        vitq.vq_absorb_thresholds(0.05, s_w, bias, [0.0], 4)
    assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_STEP")
