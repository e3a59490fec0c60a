"""GPU: vq_attention_block_static (the entry point that allocates nothing: intermediates in the
library's own static device array) against vq_attention_block with a caller workspace, on two calls
in a row, the second with a smaller input; plus the oracle for the first call and the size limit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq, workloads as wl
from tests.gpu_util import assert_fp32_close, dev, device_weights, quantized_weights


def _case(name, images, sharp=True, bits=4):
    dims = wl.block_dims(name)
    D, N = dims["D"], dims["N"]
    B = len(images)
    st = wl.block_steps(name, sharp, bits, bits)
    wts = quantized_weights(wl.block_weights(name, sharp=sharp), bits)
    wd = device_weights(wts, bits)
    tokens = wl.block_tokens(name, images).reshape(B * N, D)
    xq = vitq.QMat.empty(B * N, D, bits)
    vitq.vq_quantize(dev(tokens), st["s_x"], None, xq)
    desc = vitq.make_block_desc(dims, bits, bits, 4, wd, st)
    return dict(dims=dims, B=B, st=st, wts=wts, wd=wd, tokens=tokens, xq=xq, desc=desc)


def _both(c):
    B, N, D = c["B"], c["dims"]["N"], c["dims"]["D"]
    ws = torch.empty(max(vitq.vq_attention_block_workspace(c["desc"], B), 256), dtype=torch.uint8, device="cuda")
    y_ws = torch.full((B * N, D), -9.0, dtype=torch.float32, device="cuda")
    y_st = torch.full((B * N, D), -7.0, dtype=torch.float32, device="cuda")
    vitq.vq_attention_block(c["desc"], c["xq"], B, y_ws, ws)
    vitq.vq_attention_block_static(c["desc"], c["xq"], B, y_st)
    torch.cuda.synchronize()
    return y_ws.cpu().numpy(), y_st.cpu().numpy()


def test_static_scratch_entry_matches_workspace_entry_twice_second_smaller():
    big = _case("tiny_block", list(range(wl.BLOCKS["tiny_block"]["batch"])))
    small = _case("tiny_block", [1])
    for c, what in ((big, "first call"), (small, "second, smaller call")):
        y_ws, y_st = _both(c)
        assert np.array_equal(y_ws, y_st), what + ": static-scratch output differs from the workspace entry point's"
        xq = vqo.quantize(c["tokens"], c["st"]["s_x"], 4)
        ref = vqo.attention_block(xq, c["B"], c["dims"], c["wts"], c["st"], bits_a=4, bits_p=4, dumps=False)
        assert_fp32_close(y_st, ref["y"], what + " against the oracle")


def test_static_scratch_entry_attention_only_chain_and_other_shape():
    for images in ([0, 1, 2], [2]):
        c = _case("vit_s_attn", images)
        y_ws, y_st = _both(c)
        assert np.array_equal(y_ws, y_st)


def test_static_scratch_entry_rejects_what_does_not_fit():
    c = _case("tiny_block", [0])
    dims = c["dims"]
    # a batch whose intermediates exceed the static array: rejected on the host, nothing launched
    B = 1
    while vitq.vq_attention_block_workspace(c["desc"], B) <= (16 << 20):
        B *= 2
    xq = vitq.QMat.empty(B * dims["N"], dims["D"], 4)
    y = torch.full((B * dims["N"], dims["D"]), 3.0, dtype=torch.float32, device="cuda")
    with pytest.raises(vitq.VitqError) as e:
        vitq.vq_attention_block_static(c["desc"], xq, B, y)
    assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_WORKSPACE")
    torch.cuda.synchronize()
    assert float(y.min()) == 3.0 and float(y.max()) == 3.0
