"""GPU parity: vq_vit_block (pre-LayerNorm block on the fp32 residual stream) against the CPU
oracle chain -- every quantized intermediate byte-identical, x1 and y within 1e-5 rel / 1e-6 abs
(in fact expected identical)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import vqo
from paper_2504_18547_amd import vitq, workloads as wl
from tests.gpu_util import assert_fp32_close, dev, device_weights, preln_case, storage_of


def _run(name, images, sharp, bits_w, bits_a, prepack=False, dumps=True):
    c = preln_case(name, sharp, bits_w, bits_a, images)
    dims, st, wts, ln, x = c["dims"], c["st"], c["wts"], c["ln"], c["x"]
    D, N, hidden = dims["D"], dims["N"], dims["hidden"]
    B = len(images)
    sa = storage_of(bits_a)
    wd = device_weights(wts, bits_w, prepack=prepack)
    dump_t = {}
    if dumps:
        dump_t["o"] = torch.zeros((B * N, D * sa // 8), dtype=torch.uint8, device="cuda")
        dump_t["x2"] = torch.zeros((B * N, D * sa // 8), dtype=torch.uint8, device="cuda")
        dump_t["h"] = torch.zeros((B * N, hidden * sa // 8), dtype=torch.uint8, device="cuda")
    blk = vitq.make_block_desc(dims, bits_a, bits_a, sa, wd, st, dump_t)
    lnd = {k: dev(v) for k, v in ln.items() if k != "eps"}
    lnd["eps"] = ln["eps"]
    xq_t = torch.zeros((B * N, D * sa // 8), dtype=torch.uint8, device="cuda") if dumps else None
    x1_t = torch.zeros((B * N, D), dtype=torch.float32, device="cuda") if dumps else None
    desc = vitq.make_preln_desc(blk, lnd, xq_t, x1_t)
    ws = torch.empty(vitq.vq_vit_block_workspace(desc, B), dtype=torch.uint8, device="cuda")
    xd = dev(x)
    y = torch.full((B * N, D), -9.0, dtype=torch.float32, device="cuda")
    vitq.vq_vit_block(desc, xd, B, y, ws)
    torch.cuda.synchronize()
    ref = vqo.vit_block_preln(x, B, dims, wts, st, ln, bits_a=bits_a, bits_p=bits_a)
    what = "%s w%da%d" % (name, bits_w, bits_a)
    if dumps:
        assert np.array_equal(vqo.unpack(xq_t.cpu().numpy(), D, sa), ref["xq"]), what + ": LN1 levels differ"
        assert np.array_equal(vqo.unpack(dump_t["o"].cpu().numpy(), D, sa), ref["o"]), what + ": O differs"
        assert np.array_equal(x1_t.cpu().numpy(), ref["x1"]), what + ": x1 differs"
        assert np.array_equal(vqo.unpack(dump_t["x2"].cpu().numpy(), D, sa), ref["x2"]), what + ": LN2 levels differ"
        assert np.array_equal(vqo.unpack(dump_t["h"].cpu().numpy(), hidden, sa), ref["h"]), what + ": H differs"
    got = y.cpu().numpy()
    assert_fp32_close(got, ref["y"], what + " y")
    assert np.array_equal(got, ref["y"]), "fp32 outputs are expected to be identical"
    assert torch.equal(xd.cpu(), torch.from_numpy(x)), "the input stream must not be modified"
    return got, ref


@pytest.mark.parametrize("bits_w,bits_a,prepack", [(4, 4, False), (4, 4, True), (3, 4, False), (2, 4, True),
                                                   (8, 8, False)])
@pytest.mark.parametrize("sharp", [False, True])
def test_tiny_block(bits_w, bits_a, prepack, sharp):
    got, ref = _run("tiny_block", [0, 1], sharp, bits_w, bits_a, prepack=prepack)
    assert np.abs(ref["y"] - ref["x1"]).max() > 0.05


def test_long_rows():
    _run("tiny_long", [0, 1], True, 4, 4)


def test_dumps_do_not_change_the_result():
    a, _ = _run("tiny_block", [0, 1], True, 4, 4, dumps=True)
    b, _ = _run("tiny_block", [0, 1], True, 4, 4, dumps=False)
    assert np.array_equal(a, b)


def test_vit_b_block_reduced_batch():
    _run("vit_b_block", [0, 1, 2], True, 4, 4, dumps=True)


def test_missing_layernorm_parameters_are_rejected():
    c = preln_case("tiny_block", True, 4, 4, [0])
    dims, st = c["dims"], c["st"]
    wd = device_weights(c["wts"], 4)
    blk = vitq.make_block_desc(dims, 4, 4, 4, wd, st)
    lnd = {k: dev(v) for k, v in c["ln"].items() if k != "eps"}
    lnd["eps"] = c["ln"]["eps"]
    desc = vitq.make_preln_desc(blk, lnd)
    ws = torch.empty(vitq.vq_vit_block_workspace(desc, 1), dtype=torch.uint8, device="cuda")
    x = dev(c["x"])
    desc.ln2_beta = None
    y = torch.zeros_like(x)
    with pytest.raises(vitq.VitqError) as e:
        vitq.vq_vit_block(desc, x, 1, y, ws)
    assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_NULL")
    torch.cuda.synchronize()
    assert torch.all(y == 0)


def _layer(c, bits_w, bits_a, keep):
    """Descriptor of one encoder layer from a preln_case; the device tensors go into `keep` (the
    descriptor only holds raw pointers)."""
    sa = storage_of(bits_a)
    wd = device_weights(c["wts"], bits_w)
    lnd = {k: dev(v) for k, v in c["ln"].items() if k != "eps"}
    lnd["eps"] = c["ln"]["eps"]
    blk = vitq.make_block_desc(c["dims"], bits_a, bits_a, sa, wd, c["st"])
    keep.append((wd, lnd, blk))
    return vitq.make_preln_desc(blk, lnd)


def test_encoder_of_three_layers_and_in_place_stream():
    images = [0, 1]
    cases = [preln_case("tiny_block", sharp, 4, 4, images) for sharp in (False, True, False)]
    dims = cases[0]["dims"]
    B, N, D = len(images), dims["N"], dims["D"]
    x = cases[0]["x"]
    h = x
    for c in cases:                                   # the oracle, layer by layer
        h = vqo.vit_block_preln(h, B, dims, c["wts"], c["st"], c["ln"], bits_a=4, bits_p=4)["y"]
    keep = []
    descs = [_layer(c, 4, 4, keep) for c in cases]
    ws = torch.empty(vitq.vq_vit_encoder_workspace(descs, B), dtype=torch.uint8, device="cuda")
    xd = dev(x)
    y = torch.full((B * N, D), -9.0, dtype=torch.float32, device="cuda")
    vitq.vq_vit_encoder(descs, xd, B, y, ws)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), h)
    assert torch.equal(xd.cpu(), torch.from_numpy(x))
    # the same stack updating the stream in place
    vitq.vq_vit_encoder(descs, xd, B, xd, ws)
    torch.cuda.synchronize()
    assert np.array_equal(xd.cpu().numpy(), h)
    # one block in place as well
    xd2 = dev(x)
    vitq.vq_vit_block(descs[0], xd2, B, xd2, ws)
    torch.cuda.synchronize()
    first = vqo.vit_block_preln(x, B, dims, cases[0]["wts"], cases[0]["st"], cases[0]["ln"], bits_a=4, bits_p=4)["y"]
    assert np.array_equal(xd2.cpu().numpy(), first)


def test_partly_overlapping_streams_and_mismatched_layers_are_rejected():
    c = preln_case("tiny_block", False, 4, 4, [0, 1])
    dims = c["dims"]
    B, N, D = 2, dims["N"], dims["D"]
    keep = []
    desc = _layer(c, 4, 4, keep)
    ws = torch.empty(vitq.vq_vit_block_workspace(desc, B), dtype=torch.uint8, device="cuda")
    buf = torch.zeros((B * N + 4, D), dtype=torch.float32, device="cuda")
    with pytest.raises(vitq.VitqError) as e:
        vitq.vq_vit_block(desc, buf[:B * N], B, buf[4:], ws)
    assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_STRIDE")
    other = _layer(preln_case("tiny_long", False, 4, 4, [0]), 4, 4, keep)
    with pytest.raises(vitq.VitqError) as e:
        vitq.vq_vit_encoder_workspace([desc, other], B)
    assert e.value.status == vitq.STATUS_NAMES.index("VQ_ERR_SHAPE")
