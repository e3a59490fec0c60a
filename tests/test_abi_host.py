"""The C-ABI library loads, exports what include/vitq.h declares, and rejects bad arguments on
the host before touching the GPU (CPU only: no call here reaches a launch)."""
import ctypes as C

import numpy as np
import os
import re

import pytest

from oracle import vqo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2504_18547_amd import vitq
    if not os.path.exists(vitq.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return vitq.lib()


def test_every_declared_symbol_is_exported(lib):
    from paper_2504_18547_amd import vitq
    with open(os.path.join(ROOT, "include", "vitq.h")) as f:
        src = f.read()
    declared = set(re.findall(r"\b(vq_[a-z_0-9]+)\s*\(", src))
    assert declared == set(vitq.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layout_matches_header(lib, tmp_path):
    import subprocess
    from paper_2504_18547_amd import vitq
    src = tmp_path / "sz.c"
    src.write_text('#include "vitq.h"\n#include <stdio.h>\n#include <stddef.h>\n'
                   'int main(){printf("%zu %zu %zu %zu %zu\\n", sizeof(vq_qmat), sizeof(vq_block_desc),'
                   'offsetof(vq_block_desc, w_fc2), offsetof(vq_block_desc, s_x), offsetof(vq_block_desc, dump_qkv));}')
    exe = tmp_path / "sz"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(v) for v in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()]
    d = vitq.vq_block_desc
    assert got == [C.sizeof(vitq.vq_qmat), C.sizeof(d), d.w_fc2.offset, d.s_x.offset, d.dump_qkv.offset]


def test_status_strings(lib):
    from paper_2504_18547_amd import vitq
    for i in range(len(vitq.STATUS_NAMES)):
        assert len(vitq.status_string(i)) > 0
    assert vitq.status_string(0) == "ok"


def _qm(vitq, rows, cols, bits, sb, unsigned=0, stride=None, data=0x1000):
    m = vitq.vq_qmat()
    m.data, m.bits, m.storage_bits, m.is_unsigned = data, bits, sb, unsigned
    m.rows, m.cols = rows, cols
    m.row_stride = stride if stride is not None else vitq.row_stride_for(cols, sb)
    return m


def test_host_side_argument_checks(lib):
    from paper_2504_18547_amd import vitq
    E = {n: i for i, n in enumerate(vitq.STATUS_NAMES)}
    x = _qm(vitq, 10, 64, 4, 4)
    w = _qm(vitq, 8, 64, 4, 4)
    fake = C.c_void_p(0x2000)
    call = lambda *a: lib.vq_linear(*a)
    ok_tail = (fake, 1, None, 0, fake, None, C.c_float(1.0), None, None)
    assert call(None, C.c_float(1.0), C.byref(w), *ok_tail) == E["VQ_ERR_NULL"]
    assert call(C.byref(x), C.c_float(1.0), C.byref(w), None, 1, None, 0, fake, None, C.c_float(1.0), None, None) == E["VQ_ERR_NULL"]
    assert call(C.byref(x), C.c_float(1.0), C.byref(w), fake, 1, None, 0, None, None, C.c_float(1.0), None, None) == E["VQ_ERR_NULL"]
    assert call(C.byref(x), C.c_float(0.0), C.byref(w), *ok_tail) == E["VQ_ERR_STEP"]
    assert call(C.byref(x), C.c_float(float("nan")), C.byref(w), *ok_tail) == E["VQ_ERR_STEP"]
    w_bad = _qm(vitq, 8, 96, 4, 4)
    assert call(C.byref(x), C.c_float(1.0), C.byref(w_bad), *ok_tail) == E["VQ_ERR_SHAPE"]
    x_bits = _qm(vitq, 10, 64, 5, 4)
    assert call(C.byref(x_bits), C.c_float(1.0), C.byref(w), *ok_tail) == E["VQ_ERR_BITS"]
    x_sb = _qm(vitq, 10, 64, 3, 3)
    assert call(C.byref(x_sb), C.c_float(1.0), C.byref(w), *ok_tail) == E["VQ_ERR_BITS"]
    x_stride = _qm(vitq, 10, 64, 4, 4, stride=24)
    assert call(C.byref(x_stride), C.c_float(1.0), C.byref(w), *ok_tail) == E["VQ_ERR_STRIDE"]
    x_small = _qm(vitq, 10, 64, 4, 4, stride=16)
    assert call(C.byref(x_small), C.c_float(1.0), C.byref(w), *ok_tail) == E["VQ_ERR_STRIDE"]
    x_align = _qm(vitq, 10, 64, 4, 4, data=0x1004)
    assert call(C.byref(x_align), C.c_float(1.0), C.byref(w), *ok_tail) == E["VQ_ERR_STRIDE"]
    x_uns = _qm(vitq, 10, 64, 4, 4, unsigned=1)
    assert call(C.byref(x_uns), C.c_float(1.0), C.byref(w), *ok_tail) == E["VQ_ERR_BITS"]
    w8 = _qm(vitq, 8, 64, 8, 8)
    assert call(C.byref(x), C.c_float(1.0), C.byref(w8), *ok_tail) == E["VQ_ERR_UNSUPPORTED"]
    assert call(C.byref(x), C.c_float(1.0), C.byref(w), fake, 1, None, 7, fake, None, C.c_float(1.0), None, None) == E["VQ_ERR_UNSUPPORTED"]
    yq = _qm(vitq, 10, 9, 4, 4)
    assert call(C.byref(x), C.c_float(1.0), C.byref(w), fake, 1, None, 0, None, None, C.c_float(1.0), C.byref(yq), None) == E["VQ_ERR_SHAPE"]
    yq = _qm(vitq, 10, 8, 4, 4)
    assert call(C.byref(x), C.c_float(1.0), C.byref(w), fake, 1, None, 0, None, None, C.c_float(-1.0), C.byref(yq), None) == E["VQ_ERR_STEP"]
    # zero rows: nothing to do, no launch
    x0 = _qm(vitq, 0, 64, 4, 4, data=None)
    assert call(C.byref(x0), C.c_float(1.0), C.byref(w), *ok_tail) == 0

    # quantize
    out = _qm(vitq, 10, 64, 4, 4)
    assert lib.vq_quantize(fake, 10, 64, 64, C.c_float(0.0), None, C.byref(out), None) == E["VQ_ERR_STEP"]
    assert lib.vq_quantize(fake, 10, 65, 65, C.c_float(1.0), None, C.byref(out), None) == E["VQ_ERR_SHAPE"]
    assert lib.vq_quantize(fake, 10, 64, 32, C.c_float(1.0), None, C.byref(out), None) == E["VQ_ERR_SHAPE"]
    assert lib.vq_quantize(None, 10, 64, 64, C.c_float(1.0), None, C.byref(out), None) == E["VQ_ERR_NULL"]
    assert lib.vq_weight_steps(fake, 4, 8, 8, 9, fake, None) == E["VQ_ERR_BITS"]
    assert lib.vq_weight_steps(None, 4, 8, 8, 4, fake, None) == E["VQ_ERR_NULL"]

    # attention matmuls
    B, H, N = 2, 3, 20
    q = _qm(vitq, B * H * N, 64, 4, 4)
    p = _qm(vitq, B * H * N, N, 4, 4, unsigned=1)
    qk = lambda *a: lib.vq_matmul_qk(*a)
    f = C.c_float
    assert qk(C.byref(q), C.byref(q), B, H, N, f(.1), f(.1), f(.125), None, None, None) == E["VQ_ERR_NULL"]
    assert qk(C.byref(q), C.byref(q), B, H, N + 1, f(.1), f(.1), f(.125), fake, None, None) == E["VQ_ERR_SHAPE"]
    assert qk(C.byref(q), C.byref(q), B, H, N, f(0), f(.1), f(.125), fake, None, None) == E["VQ_ERR_STEP"]
    q32 = _qm(vitq, B * H * N, 32, 4, 4)
    assert qk(C.byref(q32), C.byref(q32), B, H, N, f(.1), f(.1), f(.125), fake, None, None) == E["VQ_ERR_UNSUPPORTED"]
    p_signed = _qm(vitq, B * H * N, N, 4, 4, unsigned=0)
    assert qk(C.byref(q), C.byref(q), B, H, N, f(.1), f(.1), f(.125), None, C.byref(p_signed), None) == E["VQ_ERR_BITS"]
    big = _qm(vitq, 600, 64, 4, 4)
    assert qk(C.byref(big), C.byref(big), 1, 1, 600, f(.1), f(.1), f(.125), fake, None, None) == E["VQ_ERR_UNSUPPORTED"]
    pv = lambda *a: lib.vq_matmul_pv(*a)
    assert pv(C.byref(p), C.byref(q), B, H, N, f(1 / 15), f(.1), None, None, f(1.0), None, None) == E["VQ_ERR_NULL"]
    assert pv(C.byref(p_signed), C.byref(q), B, H, N, f(1 / 15), f(.1), fake, None, f(1.0), None, None) == E["VQ_ERR_BITS"]
    oq = _qm(vitq, B * N, H * 64, 4, 4)
    assert pv(C.byref(p), C.byref(q), B, H, N, f(1 / 15), f(.1), None, None, f(0.0), C.byref(oq), None) == E["VQ_ERR_STEP"]

    # block
    d = vitq.vq_block_desc()
    n = C.c_size_t()
    assert lib.vq_attention_block_workspace(C.byref(d), 1, C.byref(n)) == E["VQ_ERR_SHAPE"]
    d.D, d.H, d.N, d.hidden, d.bits_a, d.bits_p, d.storage_a = 128, 2, 50, 256, 4, 4, 4
    assert lib.vq_attention_block_workspace(C.byref(d), 2, C.byref(n)) == 0
    # Q,K,V (3*B*H*N rows of 32 B) + O + X2 (B*N rows of 64 B) + H (B*N rows of 128 B), 256-aligned
    assert n.value == 19200 + 6400 + 6400 + 12800
    d.H = 4
    assert lib.vq_attention_block_workspace(C.byref(d), 2, C.byref(n)) == E["VQ_ERR_UNSUPPORTED"]   # head dim 32
    d.H = 2
    xq = _qm(vitq, 100, 128, 4, 4)
    assert lib.vq_attention_block(C.byref(d), C.byref(xq), 2, fake, fake, 10, None) == E["VQ_ERR_SHAPE"]  # zeroed weight descriptors


def test_host_side_argument_checks_of_the_later_entry_points(lib):
    """Absorbed mode and the 6-bit-float path: every check below returns before any GPU call."""
    from paper_2504_18547_amd import vitq
    E = {n: i for i, n in enumerate(vitq.STATUS_NAMES)}
    fake = C.c_void_p(0x2000)
    f = C.c_float
    x = _qm(vitq, 10, 64, 4, 4)
    w = _qm(vitq, 16, 64, 4, 4)
    yq = _qm(vitq, 10, 16, 4, 4)
    ab = lambda *a: lib.vq_linear_absorbed(*a)
    assert ab(C.byref(x), C.byref(w), None, None, None, C.byref(yq), None) == E["VQ_ERR_NULL"]        # no references
    assert ab(C.byref(x), C.byref(w), None, fake, None, None, None) == E["VQ_ERR_NULL"]               # no output
    assert ab(C.byref(x), C.byref(w), None, C.c_void_p(0x2002), None, C.byref(yq), None) == E["VQ_ERR_STRIDE"]
    w24 = _qm(vitq, 24, 64, 4, 4)
    yq24 = _qm(vitq, 10, 24, 4, 4)
    assert ab(C.byref(x), C.byref(w24), None, fake, None, C.byref(yq24), None) == E["VQ_ERR_UNSUPPORTED"]   # 24 channels
    yq2 = _qm(vitq, 10, 16, 2, 2)
    assert ab(C.byref(x), C.byref(w), None, fake, None, C.byref(yq2), None) == E["VQ_ERR_UNSUPPORTED"]      # 2-bit storage
    assert ab(C.byref(x), C.byref(w), None, fake, None, C.byref(_qm(vitq, 9, 16, 4, 4)), None) == E["VQ_ERR_SHAPE"]
    x0 = _qm(vitq, 0, 64, 4, 4, data=None)
    assert ab(C.byref(x0), C.byref(w), None, fake, None, C.byref(_qm(vitq, 0, 16, 4, 4, data=None)), None) == 0

    n = C.c_size_t()
    assert lib.vq_recode_e3m2_bytes(C.byref(x), C.byref(n)) == 0 and n.value == 10 * 96
    assert lib.vq_recode_e3m2_bytes(C.byref(_qm(vitq, 3, 129, 3, 4)), C.byref(n)) == 0 and n.value == 3 * 192
    assert lib.vq_recode_e3m2_bytes(C.byref(_qm(vitq, 3, 64, 8, 8)), C.byref(n)) == E["VQ_ERR_UNSUPPORTED"]
    assert lib.vq_recode_e3m2_bytes(C.byref(x), None) == E["VQ_ERR_NULL"]
    assert lib.vq_recode_e3m2(C.byref(x), fake, 10 * 96 - 1, None) == E["VQ_ERR_WORKSPACE"]
    assert lib.vq_recode_e3m2(C.byref(x), None, 10 * 96, None) == E["VQ_ERR_NULL"]
    assert lib.vq_recode_e3m2(C.byref(x), C.c_void_p(0x2008), 10 * 96, None) == E["VQ_ERR_STRIDE"]
    lin = lambda *a: lib.vq_linear_e3m2(*a)
    assert lin(fake, 10, fake, 16, 64, f(1.0), None, 1, None, fake, None) == E["VQ_ERR_NULL"]
    assert lin(fake, 10, fake, 16, 0, f(1.0), fake, 1, None, fake, None) == E["VQ_ERR_SHAPE"]
    assert lin(fake, 10, fake, 16, 64, f(0.0), fake, 1, None, fake, None) == E["VQ_ERR_STEP"]
    assert lin(C.c_void_p(0x2004), 10, fake, 16, 64, f(1.0), fake, 1, None, fake, None) == E["VQ_ERR_STRIDE"]
    assert lin(fake, 0, fake, 16, 64, f(1.0), fake, 1, None, fake, None) == 0


def test_opcount_reproduces_table1():
    """Table I: PE and MAC counts of one head (N=198, I=384, O=64)."""
    from paper_2504_18547_amd import opcount
    rows = {}
    with open(os.path.join(ROOT, "tests", "golden", "table1_counts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, _, pe, mac = line.split()
                rows[name] = (int(pe), None if mac == "-" else float(mac))
    c = opcount.head_counts(198, 384, 64)
    assert c["linear_pe"] == rows["linear"][0] and round(c["linear_mac"] / 1e6, 2) == rows["linear"][1]
    assert c["layernorm_pe"] == rows["layernorm"][0]
    assert c["delay_pe"] == rows["delay"][0]
    assert c["qk_pe"] == rows["qk_matmul"][0] and round(c["qk_mac"] / 1e6, 2) == rows["qk_matmul"][1]
    assert c["pv_pe"] == rows["pv_matmul"][0] and round(c["pv_mac"] / 1e6, 2) == rows["pv_matmul"][1]
    # block totals are sums of per-head figures
    m = opcount.block_macs(384, 6, 198)
    assert m["qkv"] == 3 * 6 * c["linear_mac"] and m["qk"] == 6 * c["qk_mac"] and m["pv"] == 6 * c["pv_mac"]
    assert round(opcount.block_ops(768, 12, 197, 3072) / 1e6, 1) == 2907.9

# ---- vq_absorb_thresholds: host arithmetic of the library against the oracle's (no GPU involved) ----
def test_library_host_helper_reproduces_the_oracle_integers():
    # vq_absorb_thresholds is host arithmetic (no GPU): written independently in the library, it
    # must land on the same integers as the oracle for every bit width
    from paper_2504_18547_amd import vitq
    rng = np.random.default_rng(40)
    for bits in (2, 3, 4, 5, 8):
        n = 64
        s_w = rng.uniform(1e-4, 0.05, n).astype(np.float32)
        bias = rng.normal(0, 0.3, n).astype(np.float32)
        s_y = rng.uniform(0.01, 0.5, n).astype(np.float32)
        s_x = np.float32(rng.uniform(0.01, 0.2))
        for b, sy in ((bias, s_y), (None, s_y[:1])):
            got = vitq.vq_absorb_thresholds(s_x, s_w, b, sy, bits)
            want = vqo.absorb(s_x, s_w, b, sy, bits, Nout=n)
            assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])


def test_library_host_helper_rejects_bad_arguments():
    from paper_2504_18547_amd import vitq
    s_w = np.float32([0.01, 0.02])
    code = lambda name: vitq.STATUS_NAMES.index(name)
    for bits in (1, 9):
        with pytest.raises(vitq.VitqError) as e:
            vitq.vq_absorb_thresholds(0.1, s_w, None, [0.1], bits)
        assert e.value.status == code("VQ_ERR_BITS")
    for s_x, sw, sy in ((0.0, s_w, [0.1]), (0.1, np.float32([0.01, -1.0]), [0.1]), (0.1, s_w, [float("inf")]),
                        (1e-30, np.float32([1e-30, 1.0]), [0.1])):          # the last: s_x*s_w underflows to zero
        with pytest.raises(vitq.VitqError) as e:
            vitq.vq_absorb_thresholds(s_x, sw, None, sy, 4)
        assert e.value.status == code("VQ_ERR_STEP")


def test_limits_are_argument_errors_not_launch_failures(lib):
    """Sizes the kernels' 32-bit indexing cannot take are refused on the host with the codes the header lists."""
    from paper_2504_18547_amd import vitq
    E = {n: i for i, n in enumerate(vitq.STATUS_NAMES)}
    fake = C.c_void_p(0x2000)
    w = _qm(vitq, 8, 64, 4, 4)
    x_wide = _qm(vitq, 10, 64, 4, 4, stride=1 << 24)
    assert lib.vq_linear(C.byref(x_wide), C.c_float(1.0), C.byref(w), fake, 1, None, 0, fake, None, C.c_float(1.0),
                         None, None) == E["VQ_ERR_STRIDE"]
    d = vitq.vq_block_desc()
    d.D, d.H, d.N, d.hidden, d.bits_a, d.bits_p, d.storage_a = 128, 2, 512, 256, 4, 4, 4
    n = C.c_size_t()
    assert lib.vq_attention_block_workspace(C.byref(d), (1 << 13) - 1, C.byref(n)) == 0
    assert lib.vq_attention_block_workspace(C.byref(d), 1 << 13, C.byref(n)) == E["VQ_ERR_SHAPE"]      # 2^22 token rows
    # the entry point without a workspace refuses what its static array cannot hold, before any GPU call
    d.N = 50
    xq = _qm(vitq, 4000 * 50, 128, 4, 4)
    assert lib.vq_attention_block_static(C.byref(d), C.byref(xq), 4000, fake, None) == E["VQ_ERR_WORKSPACE"]


def _fake_preln_desc(vitq, D=128, H=2, N=50, hidden=256):
    """A descriptor whose every pointer is a (never dereferenced) fake address: passes all host checks."""
    d = vitq.vq_preln_desc()
    b = d.block
    b.D, b.H, b.N, b.hidden, b.bits_a, b.bits_p, b.storage_a = D, H, N, hidden, 4, 4, 4
    for nm, (r, c) in dict(w_qkv=(3 * D, D), w_proj=(D, D), w_fc1=(hidden, D), w_fc2=(D, hidden)).items():
        setattr(b, nm, _qm(vitq, r, c, 4, 4))
    for nm in ("sw_qkv", "b_qkv", "sw_proj", "b_proj", "sw_fc1", "b_fc1", "sw_fc2", "b_fc2"):
        setattr(b, nm, 0x3000)
    for nm in ("s_x", "s_q", "s_k", "s_v", "s_o", "s_x2", "s_h"):
        setattr(b, nm, 0.1)
    b.scale = 0.125
    d.ln1_gamma = d.ln1_beta = d.ln2_gamma = d.ln2_beta = 0x3000
    d.ln_eps = 1e-6
    return d


def test_encoder_checks_every_layer_before_the_first_launch(lib):
    """A bad descriptor in a later layer is reported by its own code, and nothing has been enqueued by
    then (there is no GPU here: an attempted launch of layer 0 would come back as VQ_ERR_HIP instead)."""
    from paper_2504_18547_amd import vitq
    E = {n: i for i, n in enumerate(vitq.STATUS_NAMES)}
    good, bad = _fake_preln_desc(vitq), _fake_preln_desc(vitq)
    bad.block.s_h = float("nan")
    layers = (vitq.vq_preln_desc * 3)()
    for i, dsc in enumerate((good, good, bad)):
        C.memmove(C.byref(layers[i]), C.byref(dsc), C.sizeof(vitq.vq_preln_desc))
    n = C.c_size_t()
    assert lib.vq_vit_encoder_workspace(layers, 3, 2, C.byref(n)) == 0
    x, y, ws = C.c_void_p(0x10000), C.c_void_p(0x200000), C.c_void_p(0x400000)
    assert lib.vq_vit_encoder(layers, 3, x, 2, y, ws, n.value, None) == E["VQ_ERR_STEP"]
    bad.block.s_h = 0.1
    bad.ln2_beta = None
    C.memmove(C.byref(layers[2]), C.byref(bad), C.sizeof(vitq.vq_preln_desc))
    assert lib.vq_vit_encoder(layers, 3, x, 2, y, ws, n.value, None) == E["VQ_ERR_NULL"]
    assert lib.vq_vit_encoder(layers, 3, x, 2, y, ws, n.value - 1, None) == E["VQ_ERR_WORKSPACE"]
