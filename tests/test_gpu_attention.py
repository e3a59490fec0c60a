"""GPU parity: vq_matmul_qk and vq_matmul_pv against the CPU oracle (bit-exact scores, levels and
accumulators; fp32 within 1e-5 rel / 1e-6 abs)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq
from tests.gpu_util import assert_fp32_close, dev, from_qmat, to_qmat


def _heads(rng, B, H, N, bits, spread=1.0):
    lo, hi = vqo.qrange(bits)
    def draw():
        v = np.rint(rng.standard_normal((B, H, N, 64)) * (hi / 2.5) * spread)
        return np.clip(v, lo, hi).astype(np.int8)
    return draw(), draw(), draw()


def _check_qk(q, k, s_q, s_k, bits, bits_p, p_storage=None):
    B, H, N, _ = q.shape
    qd, kd = to_qmat(q.reshape(-1, 64), bits), to_qmat(k.reshape(-1, 64), bits)
    s_acc = torch.full((B * H * N, N), -9, dtype=torch.int32, device="cuda")
    p = vitq.QMat.empty(B * H * N, N, bits_p, storage_bits=p_storage, unsigned=True)
    p.data.fill_(0xFF)
    vitq.vq_matmul_qk(qd, kd, B, H, N, s_q, s_k, 0.125, s_acc, p)
    torch.cuda.synchronize()
    ref = vqo.matmul_qk(q, k, s_q, s_k, np.float32(0.125), bits_p)
    assert np.array_equal(s_acc.cpu().numpy().reshape(B, H, N, N), ref["s_acc"]), "scores differ"
    got = from_qmat(p).reshape(B, H, N, N)
    assert np.array_equal(got, ref["p"]), "P levels differ (%d of %d)" % ((got != ref["p"]).sum(), got.size)
    assert np.array_equal(p.data.cpu().numpy(), vqo.pack(ref["p"].reshape(-1, N), p.storage_bits))
    return ref


@pytest.mark.parametrize("B,H,N", [(2, 3, 197), (1, 2, 198), (3, 1, 5), (1, 1, 1), (2, 2, 37), (1, 2, 208),
                                   (1, 1, 577), (1, 2, 209)])
def test_qk_4bit(B, H, N):
    rng = np.random.default_rng(B * 100 + H * 10 + N)
    q, k, _ = _heads(rng, B, H, N, 4)
    ref = _check_qk(q, k, np.float32(0.62), np.float32(0.58), 4, 4)
    if N >= 37:
        assert ref["p"].max() >= 5 and (ref["p"] > 0).mean() > 0.003     # not degenerate


@pytest.mark.parametrize("N", [197, 40, 577])
def test_qk_8bit_operands_and_8bit_levels(N):
    rng = np.random.default_rng(900 + N)
    q, k, _ = _heads(rng, 1, 2, N, 8)
    ref = _check_qk(q, k, np.float32(0.036), np.float32(0.034), 8, 8)
    assert ref["p"].max() > 100
    _check_qk(q, k, np.float32(0.036), np.float32(0.034), 8, 4, p_storage=8)


def test_qk_extremes_ties_and_uniform_rows():
    N = 197
    q = np.full((1, 1, N, 64), -8, np.int8)
    k = np.full((1, 1, N, 64), -8, np.int8)
    ref = _check_qk(q, k, np.float32(0.3), np.float32(0.3), 4, 4)       # uniform rows: all levels 0
    assert ref["s_acc"].max() == 4096 and ref["p"].max() == 0
    k2 = np.zeros((1, 1, N, 64), np.int8)
    k2[0, 0, 3, :] = 7
    k2[0, 0, 100, :] = 7                                               # two equal maxima: exact tie -> 7
    q2 = np.full((1, 1, N, 64), 7, np.int8)
    ref = _check_qk(q2, k2, np.float32(0.9), np.float32(0.9), 4, 4)
    assert ref["p"][0, 0, 0, 3] == 7 and ref["p"][0, 0, 0, 100] == 7 and ref["p"][0, 0, 0].sum() == 14
    k3 = np.zeros((1, 1, N, 64), np.int8)
    k3[0, 0, 50, :] = 7                                                # one-hot
    ref = _check_qk(q2, k3, np.float32(0.9), np.float32(0.9), 4, 4)
    assert ref["p"][0, 0, 0, 50] == 15 and ref["p"][0, 0, 0].sum() == 15


def test_qk_small_alpha_rows_beyond_the_exponential_table():
    """With small steps the exponential has not reached 0 where the kernel's table ends: rows whose
    score spread exceeds the table are computed directly, the others read it."""
    rng = np.random.default_rng(321)
    for N in (5, 24):
        q, k, _ = _heads(rng, 2, 2, N, 4, spread=0.5)  # spreads of a few hundred: inside the table
        q[0, 0, 1, :] = 7
        k[0, 0, 2, :] = 7
        k[0, 0, 3, :] = -8                              # row 1 of head (0,0): spread 64*7*15 = 6720
        q[1, 1, 4, :] = -8
        k[1, 1, 0, :] = -8
        k[1, 1, N - 1, :] = 7                           # spread 64*8*15 = 7680
        ref = _check_qk(q, k, np.float32(0.2), np.float32(0.2), 4, 4)
        spread = ref["s_acc"].max(axis=-1) - ref["s_acc"].min(axis=-1)
        assert (spread >= 2048).sum() >= 2 and (spread < 2048).sum() >= 2 * N
        assert len(np.unique(ref["p"])) >= 3


def _check_pv(p, v, s_p, s_v, s_o, bits, bits_p, p_storage=None, bits_o=None):
    B, H, N, _ = v.shape
    pd = to_qmat(p.reshape(-1, N), bits_p, storage_bits=p_storage)
    vd = to_qmat(v.reshape(-1, 64), bits)
    o_acc = torch.full((B * H * N, 64), -9, dtype=torch.int32, device="cuda")
    o = torch.full((B * N, H * 64), -9.0, dtype=torch.float32, device="cuda")
    bits_o = bits if bits_o is None else bits_o
    oq = vitq.QMat.empty(B * N, H * 64, bits_o, storage_bits=bits)
    vitq.vq_matmul_pv(pd, vd, B, H, N, s_p, s_v, o_acc, o, s_o, oq)
    torch.cuda.synchronize()
    ref = vqo.matmul_pv(p, v, s_p, s_v, s_o=s_o, bits_o=bits_o)
    assert np.array_equal(o_acc.cpu().numpy().reshape(B, H, N, 64), ref["o_acc"]), "accumulators differ"
    assert_fp32_close(o.cpu().numpy(), ref["o"], "o")
    assert np.array_equal(from_qmat(oq), ref["oq"]), "requantized O differs"
    return ref


@pytest.mark.parametrize("B,H,N", [(2, 3, 197), (1, 2, 198), (3, 1, 5), (1, 1, 1), (1, 2, 64), (1, 1, 577)])
def test_pv_4bit(B, H, N):
    rng = np.random.default_rng(B * 100 + H * 10 + N + 1)
    _, _, v = _heads(rng, B, H, N, 4)
    p = rng.integers(0, 16, (B, H, N, N)).astype(np.uint8)
    ref = _check_pv(p, v, np.float32(1) / np.float32(15), np.float32(0.4), np.float32(3.0 if N > 50 else 0.5), 4, 4)
    if N > 50:
        assert len(np.unique(ref["oq"])) >= 6


@pytest.mark.parametrize("N", [197, 30, 577])
def test_pv_8bit_levels(N):
    rng = np.random.default_rng(77 + N)
    _, _, v = _heads(rng, 1, 2, N, 8)
    p = rng.integers(0, 256, (1, 2, N, N)).astype(np.uint8)
    p[0, 0, 0, :] = 255
    p[0, 0, 1 % N, :] = 0
    _check_pv(p, v, np.float32(1) / np.float32(255), np.float32(0.02), np.float32(0.7), 8, 8)
    p4 = (p >> 4).astype(np.uint8)
    _check_pv(p4, v, np.float32(1) / np.float32(15), np.float32(0.02), np.float32(0.7), 8, 4, p_storage=8)


@pytest.mark.parametrize("bits,bits_o", [(4, 3), (4, 2), (8, 5), (8, 7)])
def test_pv_output_levels_narrower_than_their_storage(bits, bits_o):
    rng = np.random.default_rng(500 + bits_o)
    _, _, v = _heads(rng, 1, 2, 100, bits)
    p = rng.integers(0, 16, (1, 2, 100, 100)).astype(np.uint8)
    s_v = np.float32(0.4 if bits == 4 else 0.02)
    ref = _check_pv(p, v, np.float32(1) / np.float32(15), s_v, np.float32(6.0 / (1 << bits_o)), bits, 4,
                    p_storage=bits, bits_o=bits_o)
    lo, hi = vqo.qrange(bits_o)
    assert ref["oq"].min() == lo and ref["oq"].max() == hi


def test_pv_one_hot_rows_and_extremes():
    rng = np.random.default_rng(78)
    N = 197
    _, _, v = _heads(rng, 1, 2, N, 4)
    perm = rng.permutation(N)
    p = np.zeros((1, 2, N, N), np.uint8)
    p[:, :, np.arange(N), perm] = 15
    ref = _check_pv(p, v, np.float32(1) / np.float32(15), np.float32(1.0), np.float32(1.0), 4, 4)
    assert np.array_equal(ref["o_acc"], 15 * v[:, :, perm, :].astype(np.int32))
    p = np.full((1, 2, N, N), 15, np.uint8)
    v = np.full((1, 2, N, 64), -8, np.int8)
    ref = _check_pv(p, v, np.float32(1) / np.float32(15), np.float32(0.1), np.float32(10.0), 4, 4)
    assert ref["o_acc"].min() == -8 * 15 * N
