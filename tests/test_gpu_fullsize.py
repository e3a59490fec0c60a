"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times: the
whole batch runs on the GPU, and sampled images (images are independent) are recomputed one by
one by the CPU oracle and compared in full."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq, workloads as wl
from tests.gpu_util import assert_fp32_close, dev, device_weights, quantized_weights, storage_of


def _full_batch(name, sharp, bits_w, bits_a, sample, prepack=False):
    dims = wl.block_dims(name)
    D, H, N, hidden = dims["D"], dims["H"], dims["N"], dims["hidden"]
    B = wl.BLOCKS[name]["batch"]
    sa = storage_of(bits_a)
    st = wl.block_steps(name, sharp, bits_w, bits_a)
    wts = quantized_weights(wl.block_weights(name, sharp=sharp), bits_w)
    wd = device_weights(wts, bits_w, prepack=prepack)
    xq = vitq.QMat.empty(B * N, D, bits_a)
    chunk = 32
    for b0 in range(0, B, chunk):                       # stage the tokens in chunks (host memory)
        imgs = list(range(b0, min(B, b0 + chunk)))
        t = dev(wl.block_tokens(name, imgs).reshape(len(imgs) * N, D))
        part = vitq.QMat(xq.data[b0 * N:(b0 + len(imgs)) * N], D, bits_a, sa)
        vitq.vq_quantize(t, st["s_x"], None, part)
    desc = vitq.make_block_desc(dims, bits_a, bits_a, sa, wd, st)
    ws = torch.empty(vitq.vq_attention_block_workspace(desc, B), dtype=torch.uint8, device="cuda")
    y = torch.empty((B * N, D), dtype=torch.float32, device="cuda")
    vitq.vq_attention_block(desc, xq, B, y, ws)
    torch.cuda.synchronize()
    for i in sample:
        tok = wl.block_tokens(name, [i]).reshape(N, D)
        xq_ref = vqo.quantize(tok, st["s_x"], bits_a)
        got_x = vqo.unpack(xq.data[i * N:(i + 1) * N].cpu().numpy(), D, sa)
        assert np.array_equal(got_x, xq_ref)
        ref = vqo.attention_block(xq_ref, 1, dims, wts, st, bits_a=bits_a, bits_p=bits_a, dumps=False)
        got = y[i * N:(i + 1) * N].cpu().numpy()
        assert_fp32_close(got, ref["y"], "%s image %d" % (name, i))
        assert np.array_equal(got, ref["y"]), "fp32 outputs are expected to be identical"


@pytest.mark.parametrize("sharp", [False, True])
def test_config4_vit_b_block_b256_w4a4(sharp):
    _full_batch("vit_b_block", sharp, 4, 4, sample=[0, 131, 255])


@pytest.mark.parametrize("bits_w,bits_a", [(3, 4), (2, 4), (8, 8)])
def test_config4_other_bit_widths(bits_w, bits_a):
    _full_batch("vit_b_block", True, bits_w, bits_a, sample=[77, 255])


def test_config4_expanded_weight_kernels():
    _full_batch("vit_b_block", True, 4, 4, sample=[200], prepack=True)


def test_config2_vit_s_attention_b64():
    _full_batch("vit_s_attn", True, 4, 4, sample=[0, 63])


def test_config3_vit_b_block_b128():
    _full_batch("vit_b_block_b128", True, 4, 4, sample=[127])


@pytest.mark.parametrize("bits_w,bits_a", [(4, 4), (8, 8)])
def test_config5_vit_l_577_b64(bits_w, bits_a):
    _full_batch("vit_l_577_block", True, bits_w, bits_a, sample=[63])


def test_config4_full_batch_with_qk_layernorm():
    """Table I's attention topology (per-head LayerNorm quantizers on Q and K, fused into the QKV
    epilogue) on the whole B = 256 batch; sampled images recomputed by the oracle."""
    name, bits = "vit_b_block", 4
    dims = wl.block_dims(name)
    D, N = dims["D"], dims["N"]
    B = wl.BLOCKS[name]["batch"]
    lo, hi = vqo.qrange(bits)
    st = dict(wl.block_steps(name, True, bits, bits))
    st["s_q"] = st["s_k"] = np.float32(3.0 / hi)
    wts = quantized_weights(wl.block_weights(name, sharp=True), bits)
    wd = device_weights(wts, bits)
    rng = np.random.default_rng(99)
    ln = dict(gamma=(1 + 0.2 * rng.standard_normal(2 * D)).astype(np.float32),
              beta=(0.1 * rng.standard_normal(2 * D)).astype(np.float32), eps=np.float32(1e-6))
    xq = vitq.QMat.empty(B * N, D, bits)
    for b0 in range(0, B, 32):
        imgs = list(range(b0, min(B, b0 + 32)))
        part = vitq.QMat(xq.data[b0 * N:(b0 + len(imgs)) * N], D, bits, 4)
        vitq.vq_quantize(dev(wl.block_tokens(name, imgs).reshape(len(imgs) * N, D)), st["s_x"], None, part)
    lnd = dict(gamma=dev(ln["gamma"]), beta=dev(ln["beta"]), eps=ln["eps"])
    desc = vitq.make_block_desc(dims, bits, bits, 4, wd, st, qkln=lnd)
    ws = torch.empty(vitq.vq_attention_block_workspace(desc, B), dtype=torch.uint8, device="cuda")
    y = torch.empty((B * N, D), dtype=torch.float32, device="cuda")
    vitq.vq_attention_block(desc, xq, B, y, ws)
    torch.cuda.synchronize()
    for i in (3, 255):
        xq_ref = vqo.quantize(wl.block_tokens(name, [i]).reshape(N, D), st["s_x"], bits)
        ref = vqo.attention_block(xq_ref, 1, dims, wts, st, bits_a=bits, bits_p=bits, dumps=False, qkln=ln)
        got = y[i * N:(i + 1) * N].cpu().numpy()
        assert_fp32_close(got, ref["y"], "qk-layernorm block, image %d" % i)
        assert np.array_equal(got, ref["y"])


def test_config4_full_batch_preln_block():
    """vq_vit_block (LayerNorm quantizers, both residual adds) on the whole B = 256 batch of the fp32
    residual stream; sampled images recomputed by the oracle."""
    from tests.oracle_cases import preln_case
    name, bits = "vit_b_block", 4
    c = preln_case(name, True, bits, bits, [0])           # weights, LayerNorm parameters, steps
    dims, st, wts, ln = c["dims"], c["st"], c["wts"], c["ln"]
    D, N = dims["D"], dims["N"]
    B = wl.BLOCKS[name]["batch"]
    wd = device_weights(wts, bits)
    x = torch.empty((B * N, D), dtype=torch.float32, device="cuda")
    for b0 in range(0, B, 32):
        imgs = list(range(b0, min(B, b0 + 32)))
        x[b0 * N:(b0 + len(imgs)) * N] = dev(wl.block_stream(name, imgs).reshape(len(imgs) * N, D))
    blk = vitq.make_block_desc(dims, bits, bits, 4, wd, st)
    lnd = {k: dev(v) for k, v in ln.items() if k != "eps"}
    lnd["eps"] = ln["eps"]
    desc = vitq.make_preln_desc(blk, lnd)
    ws = torch.empty(vitq.vq_vit_block_workspace(desc, B), dtype=torch.uint8, device="cuda")
    y = torch.empty((B * N, D), dtype=torch.float32, device="cuda")
    vitq.vq_vit_block(desc, x, B, y, ws)
    torch.cuda.synchronize()
    for i in (1, 254):
        xi = wl.block_stream(name, [i]).reshape(N, D)
        ref = vqo.vit_block_preln(xi, 1, dims, wts, st, ln, bits_a=bits, bits_p=bits)
        got = y[i * N:(i + 1) * N].cpu().numpy()
        assert_fp32_close(got, ref["y"], "pre-LayerNorm block, image %d" % i)
        assert np.array_equal(got, ref["y"])
