"""GPU parity: vq_attention_block end to end against the CPU oracle chain, every intermediate
byte-identical, final fp32 output within 1e-5 rel / 1e-6 abs."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq, workloads as wl
from tests.gpu_util import assert_fp32_close, dev, device_weights, quantized_weights, storage_of


def run_block_gpu(name, images, sharp, bits_w, bits_a, dumps=True, x_levels=None, wts=None, prepack=False):
    """Returns (gpu outputs dict, oracle-side inputs) for the given images of a workload."""
    dims = wl.block_dims(name)
    D, H, N, hidden = dims["D"], dims["H"], dims["N"], dims["hidden"]
    B = len(images)
    st = wl.block_steps(name, sharp, bits_w, bits_a)
    sa = storage_of(bits_a)
    if wts is None:
        wts = quantized_weights(wl.block_weights(name, sharp=sharp), bits_w)
    wd = device_weights(wts, bits_w, prepack=prepack)
    tokens = wl.block_tokens(name, images).reshape(B * N, D)
    # the GPU quantizes its own input tokens with vq_quantize (parity-tested separately)
    xq = vitq.QMat.empty(B * N, D, bits_a)
    vitq.vq_quantize(dev(tokens), st["s_x"], None, xq)
    dump_t = {}
    if dumps:
        dump_t["qkv"] = torch.zeros((3 * B * H * N, 64 * sa // 8), dtype=torch.uint8, device="cuda")
        dump_t["o"] = torch.zeros((B * N, D * sa // 8), dtype=torch.uint8, device="cuda")
        if hidden:
            dump_t["x2"] = torch.zeros((B * N, D * sa // 8), dtype=torch.uint8, device="cuda")
            dump_t["h"] = torch.zeros((B * N, hidden * sa // 8), dtype=torch.uint8, device="cuda")
    desc = vitq.make_block_desc(dims, bits_a, bits_a, sa, wd, st, dump_t)
    ws = torch.empty(max(vitq.vq_attention_block_workspace(desc, B), 256), dtype=torch.uint8, device="cuda")
    y = torch.full((B * N, D), -9.0, dtype=torch.float32, device="cuda")
    vitq.vq_attention_block(desc, xq, B, y, ws)
    torch.cuda.synchronize()
    out = dict(y=y.cpu().numpy(), xq=vqo.unpack(xq.data.cpu().numpy(), D, sa))
    for k, t in dump_t.items():
        cols = {"qkv": 64, "o": D, "x2": D, "h": hidden}[k]
        out[k] = vqo.unpack(t.cpu().numpy(), cols, sa)
    return out, dict(dims=dims, st=st, wts=wts, tokens=tokens, B=B)


def compare_with_oracle(out, inp, bits_a, what=""):
    dims, st, wts, B = inp["dims"], inp["st"], inp["wts"], inp["B"]
    D, H, N, hidden = dims["D"], dims["H"], dims["N"], dims["hidden"]
    xq = vqo.quantize(inp["tokens"], st["s_x"], bits_a)
    assert np.array_equal(out["xq"], xq), what + ": quantized tokens differ"
    ref = vqo.attention_block(xq, B, dims, wts, st, bits_a=bits_a, bits_p=bits_a)
    if "qkv" in out:
        qkv = out["qkv"].reshape(3, B, H, N, 64)
        for i, nm in enumerate("qkv"):
            assert np.array_equal(qkv[i], ref[nm]), "%s: %s levels differ (%d)" % (what, nm, (qkv[i] != ref[nm]).sum())
        assert np.array_equal(out["o"], ref["o"]), "%s: O levels differ (%d)" % (what, (out["o"] != ref["o"]).sum())
        if hidden:
            assert np.array_equal(out["x2"], ref["x2"]), what + ": X2 levels differ"
            assert np.array_equal(out["h"], ref["h"]), "%s: H levels differ (%d)" % (what, (out["h"] != ref["h"]).sum())
    assert_fp32_close(out["y"], ref["y"], what + " y")
    return ref


@pytest.mark.parametrize("name", ["tiny_attn", "tiny_block"])
@pytest.mark.parametrize("sharp", [False, True])
@pytest.mark.parametrize("bits_w,bits_a,prepack", [(4, 4, False), (3, 4, False), (2, 4, False), (8, 8, False),
                                                   (4, 4, True), (3, 4, True), (2, 4, True)])
def test_tiny_blocks_all_bit_widths(name, sharp, bits_w, bits_a, prepack):
    images = list(range(wl.BLOCKS[name]["batch"]))
    out, inp = run_block_gpu(name, images, sharp, bits_w, bits_a, prepack=prepack)
    ref = compare_with_oracle(out, inp, bits_a, "%s w%da%d" % (name, bits_w, bits_a))
    if sharp:
        assert len(np.unique(ref["o"])) >= 5          # the attention output is not degenerate


@pytest.mark.parametrize("sharp", [False, True])
@pytest.mark.parametrize("bits_w,bits_a", [(4, 4), (8, 8)])
def test_long_rows_take_the_streaming_attention(bits_w, bits_a, sharp):
    """N = 230 > 208 tokens: the attention runs in its long-row (score-recomputing) form."""
    out, inp = run_block_gpu("tiny_long", [0, 1], sharp, bits_w, bits_a)
    ref = compare_with_oracle(out, inp, bits_a, "tiny_long w%da%d" % (bits_w, bits_a))
    if sharp:
        assert len(np.unique(ref["o"])) >= 5


def test_paper_head_shape_n198():
    """Table I's shape: N = 198 tokens, 384 inputs, 6 heads of 64."""
    out, inp = run_block_gpu("deit_s_table1", [0, 1], True, 4, 4, prepack=True)
    compare_with_oracle(out, inp, 4, "deit_s_table1")


def test_config2_vit_s_attention_reduced_batch():
    for sharp in (False, True):
        out, inp = run_block_gpu("vit_s_attn", [0, 1, 2], sharp, 4, 4, prepack=sharp)
        compare_with_oracle(out, inp, 4, "vit_s_attn sharp=%s" % sharp)


def test_dump_and_no_dump_runs_agree_and_are_deterministic():
    a, _ = run_block_gpu("tiny_block", [0, 1], True, 4, 4, dumps=True)
    b, _ = run_block_gpu("tiny_block", [0, 1], True, 4, 4, dumps=False)
    c, _ = run_block_gpu("tiny_block", [0, 1], True, 4, 4, dumps=False)
    assert np.array_equal(a["y"], b["y"]) and np.array_equal(b["y"], c["y"])


def test_workspace_too_small_is_rejected():
    dims = wl.block_dims("tiny_block")
    st = wl.block_steps("tiny_block", True, 4, 4)
    wd = device_weights(quantized_weights(wl.block_weights("tiny_block", sharp=True), 4), 4)
    desc = vitq.make_block_desc(dims, 4, 4, 4, wd, st)
    need = vitq.vq_attention_block_workspace(desc, 2)
    xq = vitq.QMat.empty(2 * dims["N"], dims["D"], 4)
    y = torch.zeros((2 * dims["N"], dims["D"]), device="cuda")
    ws = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(vitq.VitqError) as e:
        vitq.vq_attention_block(desc, xq, 2, y, ws)
    assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_WORKSPACE")
