"""Pins of the oracle's Q/K-LayerNorm attention variant (Sec. III, Fig. 1(b), Table I) -- CPU only."""
import numpy as np

from oracle import vqo
from paper_2504_18547_amd import workloads as wl
from tests.oracle_cases import quantized_weights


def _case(name="deit_s_table1", images=(0, 1)):
    dims = wl.block_dims(name)
    D, N = dims["D"], dims["N"]
    st = dict(wl.block_steps(name, True, 4, 4))
    st["s_q"] = st["s_k"] = np.float32(3.0 / 7)          # LayerNorm outputs: unit variance, clipped at 3 sigma
    wts = quantized_weights(wl.block_weights(name, sharp=True), 4)
    rng = np.random.default_rng(99)
    ln = dict(gamma=(1 + 0.1 * rng.standard_normal(2 * D)).astype(np.float32),
              beta=(0.05 * rng.standard_normal(2 * D)).astype(np.float32), eps=np.float32(1e-6))
    tokens = wl.block_tokens(name, list(images)).reshape(len(images) * N, D)
    xq = vqo.quantize(tokens, st["s_x"], 4)
    return dims, st, wts, ln, xq


def test_chain_equals_stage_by_stage_composition_with_table1_head_shape():
    dims, st, wts, ln, xq = _case()
    D, H, N = dims["D"], dims["H"], dims["N"]
    assert (N, D, D // H) == (198, 384, 64)               # Table I: N x O = 12,672, I x O = 24,576
    B = 2
    ref = vqo.attention_block(xq, B, dims, wts, st, qkln=ln)
    y = vqo.linear(xq, st["s_x"], wts["w_qkv"], wts["sw_qkv"], bias=wts["b_qkv"])["y"]
    for which, nm in enumerate("qk"):
        for h in range(H):
            sl = slice(which * D + h * 64, which * D + (h + 1) * 64)
            # Table I: one LayerNorm of 2 x O = 128 elements (a mean and a variance row) per Q / K head
            q = vqo.layernorm_quantize(y[:, sl], ln["gamma"][sl], ln["beta"][sl], ln["eps"],
                                       st["s_" + nm], 4)["q"]
            assert np.array_equal(ref[nm][:, h].reshape(B * N, 64), q), (nm, h)
    v = vqo.quantize(y[:, 2 * D:], st["s_v"], 4)          # V: no LayerNorm (Table I lists none)
    assert np.array_equal(ref["v"].transpose(0, 2, 1, 3).reshape(B * N, D), v)
    qk = vqo.matmul_qk(ref["q"], ref["k"], st["s_q"], st["s_k"], st["scale"], 4)
    pv = vqo.matmul_pv(qk["p"], ref["v"], np.float32(1) / np.float32(15), st["s_v"], s_o=st["s_o"], bits_o=4)
    assert np.array_equal(ref["o"], pv["oq"])
    assert len(np.unique(ref["q"])) == 16 and len(np.unique(ref["k"])) == 16 and len(np.unique(ref["o"])) >= 4


def test_scalar_activation_step_is_cancelled_by_the_layernorm():
    """Eq. 2's remark: the scalar activation step is cancelled by the subsequent LayerNorm.  With a
    zero bias, doubling s_x doubles every pre-norm value exactly, and the Q / K levels do not move."""
    dims, st, wts, ln, xq = _case(images=(0,))
    wts = dict(wts)
    wts["b_qkv"] = np.zeros_like(wts["b_qkv"])
    ln = dict(ln, eps=np.float32(0.0))
    a = vqo.attention_block(xq, 1, dims, wts, st, qkln=ln)
    st2 = dict(st, s_x=np.float32(2) * st["s_x"])
    b = vqo.attention_block(xq, 1, dims, wts, st2, qkln=ln)
    assert np.array_equal(a["q"], b["q"]) and np.array_equal(a["k"], b["k"])
    assert not np.array_equal(a["v"], b["v"])             # V has no LayerNorm: its levels do move
