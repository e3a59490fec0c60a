"""GPU parity of the experimental 6-bit-float operand path: vq_recode_e3m2 against the format's
definition (decoded here in numpy), vq_linear_e3m2 against the oracle's reordered linear (Eq. 2),
fp32 outputs bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq
from tests.gpu_util import dev, to_qmat


def _decode_e3m2(rows_of_codes, cols):
    """[rows, bytes] uint8 -> values [rows, cols] and the padding values.  A row is a sequence of 96-byte
    stages of 128 values; quarter q = 2s + h of a stage is a 192-bit string (value j at bits 6j..6j+5):
    its first 128 bits are the 16-byte piece 3h + s, its last 64 bits are half s of piece 3h + 2."""
    raw = rows_of_codes.astype(np.uint8)
    rows, nbytes = raw.shape
    stages = raw.reshape(rows, nbytes // 96, 6, 16)                      # [rows, stage, piece, byte]
    quarters = []
    for q in range(4):
        s, h = q >> 1, q & 1
        quarters.append(np.concatenate([stages[:, :, 3 * h + s, :], stages[:, :, 3 * h + 2, 8 * s:8 * s + 8]], axis=2))
    strings = np.stack(quarters, axis=2)                                 # [rows, stage, quarter, 24 bytes]
    bits = np.unpackbits(strings, axis=3, bitorder="little")             # 192 bits
    codes = (bits.reshape(rows, -1, 4, 32, 6) * (1 << np.arange(6))).sum(axis=4).reshape(rows, -1)
    s = np.where(codes & 32, -1.0, 1.0)
    e = (codes >> 2) & 7
    m = codes & 3
    val = np.where(e == 0, m / 4.0 * 2.0 ** -2, (1 + m / 4.0) * 2.0 ** (e.astype(np.float64) - 3))
    return (s * val)[:, :cols], (s * val)[:, cols:]


@pytest.mark.parametrize("bits,rows,cols", [(4, 37, 768), (3, 5, 100), (2, 3, 129), (4, 1, 1), (4, 130, 3072)])
def test_recode_matches_the_format_definition(bits, rows, cols):
    rng = np.random.default_rng(bits + rows + cols)
    lo, hi = vqo.qrange(bits)
    q = rng.integers(lo, hi + 1, size=(rows, cols)).astype(np.int8)
    q.flat[: min(16, q.size)] = np.resize(np.arange(lo, hi + 1), min(16, q.size))
    m = to_qmat(q, bits, storage_bits=4)
    out = vitq.vq_recode_e3m2(m)
    torch.cuda.synchronize()
    assert out.shape == (rows, (cols + 127) // 128 * 96)
    val, pad = _decode_e3m2(out.cpu().numpy(), cols)
    assert np.array_equal(val, q.astype(np.float64))
    assert not pad.any()


@pytest.mark.parametrize("bits_w,bits_a,M,K,Nout", [
    (4, 4, 197, 384, 1152),      # ViT-S QKV
    (4, 4, 591, 768, 768),       # three ViT-B images through the projection
    (4, 4, 300, 3072, 96),       # fc2-sized contraction
    (3, 3, 129, 200, 40),        # ragged everything, K tail inside a group of 128
    (2, 4, 64, 130, 16),
    (4, 4, 1, 64, 1),
])
def test_linear_matches_the_oracle(bits_w, bits_a, M, K, Nout):
    rng = np.random.default_rng(M + K + Nout)
    lo_a, hi_a = vqo.qrange(bits_a)
    lo_w, hi_w = vqo.qrange(bits_w)
    xq = rng.integers(lo_a, hi_a + 1, size=(M, K)).astype(np.int8)
    wq = rng.integers(lo_w, hi_w + 1, size=(Nout, K)).astype(np.int8)
    xq[0, :] = lo_a
    wq[0, :] = lo_w                                   # the largest accumulator: 64*K at 4 bits
    s_w = np.exp(rng.uniform(-7, -4, Nout)).astype(np.float32)
    bias = (rng.standard_normal(Nout) * 0.01).astype(np.float32)
    s_x = np.float32(0.31)
    x6 = vitq.vq_recode_e3m2(to_qmat(xq, bits_a, storage_bits=4))
    w6 = vitq.vq_recode_e3m2(to_qmat(wq, bits_w, storage_bits=4))
    for b, per_channel in ((bias, True), (None, False)):
        sw = s_w if per_channel else s_w[:1]
        y = torch.full((M, Nout), -7.0, dtype=torch.float32, device="cuda")
        vitq.vq_linear_e3m2(x6, M, w6, Nout, K, s_x, dev(sw), per_channel, None if b is None else dev(b), y)
        torch.cuda.synchronize()
        ref = vqo.linear(xq, s_x, wq, sw, bias=b)
        assert ref["overflow"] == 0
        assert np.array_equal(y.cpu().numpy(), ref["y"])


def test_unsupported_storage():
    q = np.zeros((4, 64), np.int8)
    with pytest.raises(vitq.VitqError) as e:
        vitq.vq_recode_e3m2(to_qmat(q, 8))
    assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_UNSUPPORTED")
