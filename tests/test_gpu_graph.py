"""GPU: the step of the benchmark (vq_quantize + vq_attention_block) captured into one HIP graph.
Every replay, with eager work and synchronizations in between, must reproduce the eager result,
which is itself checked against the CPU oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq, workloads as wl
from tests.gpu_util import assert_fp32_close, dev, device_weights, quantized_weights


@pytest.mark.parametrize("name", ["tiny_block", "tiny_long"])
def test_captured_step_replays_match_eager_and_oracle(name):
    bits = 4
    images = list(range(wl.BLOCKS[name]["batch"]))
    dims = wl.block_dims(name)
    D, N = dims["D"], dims["N"]
    B = len(images)
    st = wl.block_steps(name, True, bits, bits)
    wts = quantized_weights(wl.block_weights(name, sharp=True), bits)
    wd = device_weights(wts, bits)
    tokens_np = wl.block_tokens(name, images).reshape(B * N, D)
    tokens = dev(tokens_np)
    xq = vitq.QMat.empty(B * N, D, bits)
    desc = vitq.make_block_desc(dims, bits, bits, 4, wd, st)
    ws = torch.empty(max(vitq.vq_attention_block_workspace(desc, B), 256), dtype=torch.uint8, device="cuda")
    y = torch.zeros((B * N, D), dtype=torch.float32, device="cuda")

    def step():
        vitq.vq_quantize(tokens, st["s_x"], None, xq)
        vitq.vq_attention_block(desc, xq, B, y, ws)

    step()                                   # eager (also the first-use set-up of every kernel)
    torch.cuda.synchronize()
    eager = y.cpu().numpy().copy()
    ref = vqo.attention_block(vqo.quantize(tokens_np, st["s_x"], bits), B, dims, wts, st, bits_a=bits, bits_p=bits,
                              dumps=False)
    assert_fp32_close(eager, ref["y"], name + " eager")

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    other = torch.empty(1 << 20, device="cuda")
    for rep in range(4):
        y.fill_(-3.0)                        # eager work between the replays
        xq.data.zero_()
        other.normal_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        assert np.array_equal(got, eager), "%s: replay %d differs from the eager result" % (name, rep)
