"""Pins for the packed low-bit storage format (CPU only)."""
import numpy as np
import pytest


def test_hand_worked_bytes(vqo):
    # 4-bit: element 0 in the low nibble; two's complement
    assert vqo.pack(np.array([[1, -1]], np.int8), 4)[0, 0] == 0xF1
    assert vqo.pack(np.array([[-8, 7, 3]], np.int8), 4)[0, :2].tolist() == [0x78, 0x03]
    # 2-bit: four per byte, element 0 in the two low bits: [1,-1,0,-2] -> 10 00 11 01
    assert vqo.pack(np.array([[1, -1, 0, -2]], np.int8), 2)[0, 0] == 0b10001101
    # 8-bit
    assert vqo.pack(np.array([[-128, 127]], np.int8), 8)[0, :2].tolist() == [0x80, 0x7F]
    # unsigned 4-bit (attention levels)
    assert vqo.pack(np.array([[15, 0, 9]], np.uint8), 4)[0, :2].tolist() == [0x0F, 0x09]


@pytest.mark.parametrize("sb", [2, 4, 8])
def test_roundtrip_all_values_all_positions(vqo, sb):
    lo, hi = -(2 ** (sb - 1)), 2 ** (sb - 1) - 1
    per_byte = 8 // sb
    vals = np.arange(lo, hi + 1)
    cols = per_byte * 3 + 1                   # ragged: last byte partly used
    rows = []
    for pos in range(cols):
        for v in vals[:: max(1, len(vals) // 16)].tolist() + [lo, hi]:
            r = np.zeros(cols, np.int8)
            r[pos] = v
            rows.append(r)
    q = np.stack(rows)
    p = vqo.pack(q, sb)
    assert p.shape[1] % 16 == 0
    assert np.array_equal(vqo.unpack(p, cols, sb), q)
    used = (cols * sb + 7) // 8
    assert np.all(p[:, used:] == 0)           # pad bytes are zero
    rng = np.random.default_rng(sb)
    q = rng.integers(lo, hi + 1, (13, 45)).astype(np.int8)
    assert np.array_equal(vqo.unpack(vqo.pack(q, sb), 45, sb), q)
    u = rng.integers(0, 2 ** sb, (5, 29)).astype(np.uint8)
    assert np.array_equal(vqo.unpack(vqo.pack(u, sb), 29, sb, unsigned=True), u)


def test_three_bit_levels_live_in_nibbles(vqo):
    q = np.array([[-4, 3, -1, 2]], np.int8)
    p = vqo.pack(q, 4)
    assert p[0, :2].tolist() == [0x3C, 0x2F]
    assert np.array_equal(vqo.unpack(p, 4, 4), q)


def test_stride_too_small_is_rejected(vqo):
    with pytest.raises(ValueError):
        vqo.pack(np.zeros((2, 64), np.int8), 4, row_stride=16)
