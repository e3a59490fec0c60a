"""GPU parity of the Q/K-LayerNorm attention topology (Fig. 1(b), Table I): vq_qkv_headnorm alone and
inside vq_attention_block / vq_vit_block, against the CPU oracle -- all levels byte-identical."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq, workloads as wl
from tests.gpu_util import assert_fp32_close, dev, device_weights, preln_case, quantized_weights, storage_of


def _ln(D, seed=99):
    rng = np.random.default_rng(seed)
    return dict(gamma=(1 + 0.1 * rng.standard_normal(2 * D)).astype(np.float32),
                beta=(0.05 * rng.standard_normal(2 * D)).astype(np.float32), eps=np.float32(1e-6))


@pytest.mark.parametrize("bits,B,H,N", [(4, 2, 6, 198), (8, 1, 2, 37), (3, 3, 1, 5), (4, 1, 12, 1)])
def test_qkv_headnorm_op(bits, B, H, N):
    rng = np.random.default_rng(bits * 100 + N)
    D = 64 * H
    M = B * N
    y = (rng.standard_normal((M, 3 * D)) * rng.uniform(0.1, 3, (M, 1)) + rng.uniform(-1, 1, (M, 1))).astype(np.float32)
    y[0, :64] = 2.5                                      # a constant head
    if M > 2:
        y[2, 70] = np.inf
        y[1, 3 * D - 1] = np.nan
    ln = _ln(D)
    ln["gamma"][::5] *= -1
    lo, hi = vqo.qrange(bits)
    s_q, s_k, s_v = np.float32(3.0 / hi), np.float32(2.5 / hi), np.float32(4.0 / hi)
    sa = storage_of(bits)
    out = torch.full((3 * B * H * N, 64 * sa // 8), 0xFF, dtype=torch.uint8, device="cuda")
    vitq.vq_qkv_headnorm(dev(y), B, H, N, dev(ln["gamma"]), dev(ln["beta"]), ln["eps"], s_q, s_k, s_v, bits, sa, out)
    torch.cuda.synchronize()
    got = vqo.unpack(out.cpu().numpy(), 64, sa).reshape(3, B, H, N, 64)
    for which, step in ((0, s_q), (1, s_k)):
        for h in range(H):
            sl = slice(which * D + h * 64, which * D + (h + 1) * 64)
            ref = vqo.layernorm_quantize(y[:, sl], ln["gamma"][sl], ln["beta"][sl], ln["eps"], step, bits)["q"]
            assert np.array_equal(got[which][:, h].reshape(M, 64), ref.reshape(B, N, 64).reshape(M, 64)), (which, h)
    vref = vqo.quantize(np.nan_to_num(y[:, 2 * D:], nan=0.0) if False else y[:, 2 * D:], s_v, bits)
    assert np.array_equal(got[2].transpose(0, 2, 1, 3).reshape(M, D), vref)


def _block(name, images, bits_w, bits_a, prepack=False, steps=None):
    dims = wl.block_dims(name)
    D, H, N, hidden = dims["D"], dims["H"], dims["N"], dims["hidden"]
    B = len(images)
    sa = storage_of(bits_a)
    lo, hi = vqo.qrange(bits_a)
    st = dict(wl.block_steps(name, True, bits_w, bits_a))
    st["s_q"] = st["s_k"] = np.float32(3.0 / hi)
    for k, v in (steps or {}).items():
        st[k] = np.float32(v)
    wts = quantized_weights(wl.block_weights(name, sharp=True), bits_w)
    wd = device_weights(wts, bits_w, prepack=prepack)
    ln = _ln(D)
    tokens = wl.block_tokens(name, images).reshape(B * N, D)
    xq_ref = vqo.quantize(tokens, st["s_x"], bits_a)
    xq = vitq.QMat.empty(B * N, D, bits_a)
    vitq.vq_quantize(dev(tokens), st["s_x"], None, xq)
    dump = {"qkv": torch.zeros((3 * B * H * N, 64 * sa // 8), dtype=torch.uint8, device="cuda"),
            "o": torch.zeros((B * N, D * sa // 8), dtype=torch.uint8, device="cuda")}
    lnd = dict(gamma=dev(ln["gamma"]), beta=dev(ln["beta"]), eps=ln["eps"])
    desc = vitq.make_block_desc(dims, bits_a, bits_a, sa, wd, st, dump, qkln=lnd)
    ws = torch.empty(vitq.vq_attention_block_workspace(desc, B), dtype=torch.uint8, device="cuda")
    y = torch.full((B * N, D), -9.0, dtype=torch.float32, device="cuda")
    vitq.vq_attention_block(desc, xq, B, y, ws)
    torch.cuda.synchronize()
    ref = vqo.attention_block(xq_ref, B, dims, wts, st, bits_a=bits_a, bits_p=bits_a, qkln=ln)
    qkv = vqo.unpack(dump["qkv"].cpu().numpy(), 64, sa).reshape(3, B, H, N, 64)
    for i, nm in enumerate("qkv"):
        assert np.array_equal(qkv[i], ref[nm]), "%s: %s levels differ (%d)" % (name, nm, (qkv[i] != ref[nm]).sum())
    assert np.array_equal(vqo.unpack(dump["o"].cpu().numpy(), D, sa), ref["o"])
    assert_fp32_close(y.cpu().numpy(), ref["y"], name + " y")
    assert np.array_equal(y.cpu().numpy(), ref["y"])
    return ref


def test_table1_head_shape_n198():
    ref = _block("deit_s_table1", [0, 1], 4, 4)
    assert len(np.unique(ref["o"])) >= 4


@pytest.mark.parametrize("name,bits_w,bits_a,prepack", [("tiny_attn", 4, 4, False), ("tiny_block", 4, 4, True),
                                                        ("tiny_long", 4, 4, False),
                                                        ("tiny_block", 8, 8, False), ("tiny_attn", 2, 4, False)])
def test_small_blocks(name, bits_w, bits_a, prepack):
    _block(name, list(range(wl.BLOCKS[name]["batch"])), bits_w, bits_a, prepack)


def test_scales_too_small_to_fold():
    # s_x * s_w * 2^-8 is subnormal: the epilogue must take the unfolded scales and the explicit shift
    _block("tiny_attn", [0, 1], 4, 4, steps={"s_x": 1e-36})


def test_steps_outside_the_fused_epilogue():
    # 1/s_q beyond 2^100: the QKV linear runs in fp32 and the stand-alone head-norm kernel follows
    _block("tiny_attn", [0, 1], 4, 4, steps={"s_q": 1e-34})


def test_vit_b_block_reduced_batch():
    _block("vit_b_block", [0, 1, 2], 4, 4)


def test_preln_block_with_qk_layernorm():
    c = preln_case("tiny_block", True, 4, 4, [0, 1])
    dims, st, wts, ln, x = c["dims"], dict(c["st"]), c["wts"], c["ln"], c["x"]
    st["s_q"] = st["s_k"] = np.float32(3.0 / 7)
    D, N = dims["D"], dims["N"]
    qk = _ln(D, seed=5)
    wd = device_weights(wts, 4)
    qkd = dict(gamma=dev(qk["gamma"]), beta=dev(qk["beta"]), eps=qk["eps"])     # (kept alive: the descriptor holds raw pointers)
    blk = vitq.make_block_desc(dims, 4, 4, 4, wd, st, qkln=qkd)
    lnd = {k: dev(v) for k, v in ln.items() if k != "eps"}
    lnd["eps"] = ln["eps"]
    desc = vitq.make_preln_desc(blk, lnd)
    ws = torch.empty(vitq.vq_vit_block_workspace(desc, 2), dtype=torch.uint8, device="cuda")
    y = torch.zeros((2 * N, D), dtype=torch.float32, device="cuda")
    vitq.vq_vit_block(desc, dev(x), 2, y, ws)
    torch.cuda.synchronize()
    # the oracle chain by hand: LNQ1, attention with Q/K LayerNorm (fp32 out), +x, LNQ2, MLP, +x1
    xq = vqo.layernorm_quantize(x, ln["g1"], ln["b1"], ln["eps"], st["s_x"], 4)["q"]
    att = vqo.attention_block(xq, 2, dict(dims, hidden=0), wts, st, qkln=qk)
    l2 = vqo.layernorm_quantize(att["y"], ln["g2"], ln["b2"], ln["eps"], st["s_x2"], 4, res=x, want_sum=True)
    h = vqo.linear(l2["q"], st["s_x2"], wts["w_fc1"], wts["sw_fc1"], bias=wts["b_fc1"], act=1, s_y=st["s_h"], bits_y=4)["yq"]
    t = vqo.linear(h, st["s_h"], wts["w_fc2"], wts["sw_fc2"], bias=wts["b_fc2"])["y"]
    assert np.array_equal(y.cpu().numpy(), t + l2["sum"])


def _planted_beta(y, gamma, beta, eps, steps, bits, rng):
    """beta (Q and K channels) moved so that, for channel j, the element of token j % M sits a chosen
    distance (2^-27 .. 2^-12 levels, either side) from a comparator boundary of its (token, head) group."""
    M = y.shape[0]
    D = gamma.size // 2
    lo, hi = vqo.qrange(bits)
    beta = beta.copy()
    for j in range(2 * D):
        r = j % M
        grp = y[r, (j // 64) * 64:(j // 64) * 64 + 64]
        mu, m2 = np.float32(0), np.float32(0)
        for i in range(64):                                  # Eq. 5 in fp32, element order
            d1 = np.float32(grp[i] - mu)
            mu = np.float32(mu + np.float32(d1 / np.float32(i + 1)))
            m2 = np.float32(m2 + np.float32(d1 * np.float32(grp[i] - mu)))
        sigma = np.sqrt(float(np.float32(m2 + np.float32(64.0) * eps)) / 64.0)
        g = np.float32(np.float32(y[r, j] - mu) * gamma[j])
        step = float(steps[j // D])
        k = int(rng.integers(lo + 1, hi + 1))
        delta = float(rng.choice([-1.0, 1.0])) * 2.0 ** float(rng.uniform(-27, -12))
        beta[j] = np.float32(step * (k - 0.5 + delta) - float(g) / sigma)
    return beta


@pytest.mark.parametrize("bits", [4, 8])
def test_headnorm_op_values_planted_on_both_sides_of_the_guard(bits):
    rng = np.random.default_rng(4400 + bits)
    B, H, N = 1, 2, 96
    D, M = 64 * H, B * N
    y = (rng.standard_normal((M, 3 * D)) * rng.uniform(0.3, 3, (M, 1)) + rng.uniform(-1, 1, (M, 1))).astype(np.float32)
    ln = _ln(D)
    ln["gamma"][::7] *= -1
    lo, hi = vqo.qrange(bits)
    s_q, s_k, s_v = np.float32(3.0 / hi), np.float32(2.5 / hi), np.float32(4.0 / hi)
    ln["beta"] = _planted_beta(y, ln["gamma"], ln["beta"], ln["eps"], (s_q, s_k), bits, rng)
    sa = storage_of(bits)
    out = torch.full((3 * B * H * N, 64 * sa // 8), 0xFF, dtype=torch.uint8, device="cuda")
    vitq.vq_qkv_headnorm(dev(y), B, H, N, dev(ln["gamma"]), dev(ln["beta"]), ln["eps"], s_q, s_k, s_v, bits, sa, out)
    torch.cuda.synchronize()
    got = vqo.unpack(out.cpu().numpy(), 64, sa).reshape(3, B, H, N, 64)
    for which, step in ((0, s_q), (1, s_k)):
        for h in range(H):
            sl = slice(which * D + h * 64, which * D + (h + 1) * 64)
            ref = vqo.layernorm_quantize(y[:, sl], ln["gamma"][sl], ln["beta"][sl], ln["eps"], step, bits)["q"]
            assert np.array_equal(got[which][:, h].reshape(M, 64), ref), (which, h)


def test_fused_epilogue_values_planted_on_both_sides_of_the_guard():
    """The same through the QKV linear's epilogue: with zero QKV weights the linear's output is its bias
    (every token alike), so beta can be placed against the statistics of the bias."""
    name, bits = "tiny_attn", 4
    dims = wl.block_dims(name)
    D, H, N = dims["D"], dims["H"], dims["N"]
    B = 2
    lo, hi = vqo.qrange(bits)
    st = dict(wl.block_steps(name, True, bits, bits))
    st["s_q"] = st["s_k"] = np.float32(3.0 / hi)
    wts = quantized_weights(wl.block_weights(name, sharp=True), bits)
    rng = np.random.default_rng(77)
    wts["w_qkv"] = np.zeros_like(wts["w_qkv"])
    wts["b_qkv"] = (rng.standard_normal(3 * D) * 1.5 + 0.3).astype(np.float32)
    ybias = np.tile(wts["b_qkv"], (B * N, 1)).astype(np.float32)
    ln = _ln(D)
    ln["beta"] = _planted_beta(ybias, ln["gamma"], ln["beta"], ln["eps"], (st["s_q"], st["s_k"]), bits, rng)
    wd = device_weights(wts, bits)
    tokens = wl.block_tokens(name, list(range(B))).reshape(B * N, D)
    xq_ref = vqo.quantize(tokens, st["s_x"], bits)
    xq = vitq.QMat.empty(B * N, D, bits)
    vitq.vq_quantize(dev(tokens), st["s_x"], None, xq)
    dump = {"qkv": torch.zeros((3 * B * H * N, 64 * 4 // 8), dtype=torch.uint8, device="cuda")}
    lnd = dict(gamma=dev(ln["gamma"]), beta=dev(ln["beta"]), eps=ln["eps"])
    desc = vitq.make_block_desc(dims, bits, bits, 4, wd, st, dump, qkln=lnd)
    ws = torch.empty(vitq.vq_attention_block_workspace(desc, B), dtype=torch.uint8, device="cuda")
    y = torch.empty((B * N, D), dtype=torch.float32, device="cuda")
    vitq.vq_attention_block(desc, xq, B, y, ws)
    torch.cuda.synchronize()
    ref = vqo.attention_block(xq_ref, B, dims, wts, st, bits_a=bits, bits_p=bits, qkln=ln)
    qkv = vqo.unpack(dump["qkv"].cpu().numpy(), 64, 4).reshape(3, B, H, N, 64)
    for i, nm in enumerate("qkv"):
        assert np.array_equal(qkv[i], ref[nm]), "%s levels differ (%d)" % (nm, (qkv[i] != ref[nm]).sum())
    assert np.array_equal(y.cpu().numpy(), ref["y"])
