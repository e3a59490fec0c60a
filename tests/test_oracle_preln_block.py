"""Pins of the oracle's pre-LayerNorm block (CPU only): the chain equals a stage-by-stage
re-composition from the separately pinned routines, and images are independent."""
import numpy as np

from oracle import vqo
from paper_2504_18547_amd import workloads as wl
from tests.oracle_cases import preln_case


def test_chain_equals_stage_by_stage_composition():
    c = preln_case("tiny_block", True, 4, 4, [0, 1])
    dims, st, wts, ln, x = c["dims"], c["st"], c["wts"], c["ln"], c["x"]
    ref = vqo.vit_block_preln(x, 2, dims, wts, st, ln)
    xq = vqo.layernorm_quantize(x, ln["g1"], ln["b1"], ln["eps"], st["s_x"], 4)["q"]
    assert np.array_equal(ref["xq"], xq)
    att = vqo.attention_block(xq, 2, dict(dims, hidden=0), wts, st)        # attention + projection, fp32
    assert np.array_equal(ref["o"], att["o"])
    l2 = vqo.layernorm_quantize(att["y"], ln["g2"], ln["b2"], ln["eps"], st["s_x2"], 4, res=x, want_sum=True)
    assert np.array_equal(ref["x1"], att["y"] + x) and np.array_equal(ref["x1"], l2["sum"])
    assert np.array_equal(ref["x2"], l2["q"])
    h = vqo.linear(l2["q"], st["s_x2"], wts["w_fc1"], wts["sw_fc1"], bias=wts["b_fc1"], act=1,
                   s_y=st["s_h"], bits_y=4)["yq"]
    assert np.array_equal(ref["h"], h)
    t = vqo.linear(h, st["s_h"], wts["w_fc2"], wts["sw_fc2"], bias=wts["b_fc2"])["y"]
    assert np.array_equal(ref["y"], t + ref["x1"])
    # not degenerate: the quantizers use their range, the residual matters
    assert len(np.unique(ref["xq"])) >= 14 and len(np.unique(ref["x2"])) >= 14 and len(np.unique(ref["h"])) >= 8
    assert np.abs(ref["y"] - ref["x1"]).max() > 0.05 and np.abs(ref["x1"] - x).max() > 0.01


def test_images_are_independent():
    c = preln_case("tiny_block", True, 4, 4, [0, 1])
    dims, st, wts, ln, x = c["dims"], c["st"], c["wts"], c["ln"], c["x"]
    both = vqo.vit_block_preln(x, 2, dims, wts, st, ln, threads=2)
    n = dims["N"]
    one = vqo.vit_block_preln(x[n:], 1, dims, wts, st, ln, threads=1)
    assert np.array_equal(both["y"][n:], one["y"]) and np.array_equal(both["h"][n:], one["h"])
