"""Seeded synthetic inputs for the integerized-ViT-block workloads.

This module holds NO arithmetic of the method (no quantizer, no matmul, no softmax): it only
draws fp32 tensors with the shapes and value distributions of the benchmark configurations and
hands out the per-tensor activation steps recorded in ``workload_steps.json``.  Both the CPU
oracle (in the tests) and the GPU library are fed from here, so that they see identical inputs.

The paper evaluates a DeiT-S checkpoint on CIFAR-10 (Sec. V-A); neither is available, and
throughput does not depend on them.  These tensors stand in for them: shapes follow
DeiT-S / ViT-B / ViT-L, weights are N(0, std 0.02), biases N(0, std 0.01), tokens are N(0, 1)
followed by a LayerNorm (gamma 1, beta 0, computed in double) as the input of a pre-LN block.
"""
import json
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
STEPS_FILE = os.path.join(_HERE, "workload_steps.json")

BASE_SEED = 250418547 * 10

# name -> shapes.  "batch" is the batch the configuration is quoted on.
BLOCKS = {
    "vit_s_attn": dict(cfg=2, D=384, H=6, N=197, hidden=0, batch=64),
    "vit_b_block_b128": dict(cfg=3, D=768, H=12, N=197, hidden=3072, batch=128),
    "vit_b_block": dict(cfg=4, D=768, H=12, N=197, hidden=3072, batch=256),
    "vit_l_577_block": dict(cfg=5, D=1024, H=16, N=577, hidden=4096, batch=64),
    # small stand-ins used by the parity tests (same recipe, tiny shapes)
    "tiny_attn": dict(cfg=12, D=128, H=2, N=37, hidden=0, batch=3),
    "tiny_block": dict(cfg=13, D=128, H=2, N=50, hidden=256, batch=2),
    # more than 208 tokens at a tiny width: the long-row form of the attention kernel
    "tiny_long": dict(cfg=15, D=128, H=2, N=230, hidden=256, batch=2),
    # the paper's own per-head shape (Table I: N=198, I=384, O=64)
    "deit_s_table1": dict(cfg=14, D=384, H=6, N=198, hidden=0, batch=2),
}

LINEAR_CFG1 = dict(cfg=1, M=197, K=384, Nout=1152, bits_x=4, bits_w=4, s_x=0.1)


def seed_for(cfg_index):
    return BASE_SEED + int(cfg_index)


def linear_cfg1_inputs():
    """Config 1: the ViT-S QKV projection as a single linear (batch 1)."""
    c = LINEAR_CFG1
    rng = np.random.default_rng(seed_for(c["cfg"]))
    x = rng.standard_normal((c["M"], c["K"])).astype(np.float32)
    w = (rng.standard_normal((c["Nout"], c["K"])) * 0.02).astype(np.float32)
    b = (rng.standard_normal(c["Nout"]) * 0.01).astype(np.float32)
    return dict(x=x, w=w, bias=b, s_x=np.float32(c["s_x"]))


def block_dims(name):
    d = BLOCKS[name]
    return dict(D=d["D"], H=d["H"], N=d["N"], hidden=d["hidden"])


def block_weights(name, sharp=False):
    """fp32 weights and biases of one block.

    ``sharp=True`` draws the Q and K row blocks of the QKV weight with std
    0.08*sqrt(384/D) instead of 0.02, which gives attention logits a spread of a few units so
    that the quantized softmax has non-zero levels (with std 0.02 the softmax over 197 tokens
    is nearly uniform and every 4-bit P level is 0).
    """
    d = BLOCKS[name]
    D, hidden = d["D"], d["hidden"]
    rng = np.random.default_rng([seed_for(d["cfg"]), 1000 + int(sharp)])
    out = {}
    w_qkv = rng.standard_normal((3 * D, D)) * 0.02
    if sharp:
        w_qkv[: 2 * D] *= (0.08 * np.sqrt(384.0 / D)) / 0.02
    out["w_qkv"] = w_qkv.astype(np.float32)
    out["b_qkv"] = (rng.standard_normal(3 * D) * 0.01).astype(np.float32)
    out["w_proj"] = (rng.standard_normal((D, D)) * 0.02).astype(np.float32)
    out["b_proj"] = (rng.standard_normal(D) * 0.01).astype(np.float32)
    if hidden:
        out["w_fc1"] = (rng.standard_normal((hidden, D)) * 0.02).astype(np.float32)
        out["b_fc1"] = (rng.standard_normal(hidden) * 0.01).astype(np.float32)
        out["w_fc2"] = (rng.standard_normal((D, hidden)) * 0.02).astype(np.float32)
        out["b_fc2"] = (rng.standard_normal(D) * 0.01).astype(np.float32)
    return out


def block_tokens(name, images):
    """LayerNormed fp32 tokens [len(images), N, D].  Image i depends only on (config, i)."""
    d = BLOCKS[name]
    N, D = d["N"], d["D"]
    out = np.empty((len(images), N, D), np.float32)
    for j, i in enumerate(images):
        rng = np.random.default_rng([seed_for(d["cfg"]), 2000, int(i)])
        t = rng.standard_normal((N, D))
        mu = t.mean(axis=1, keepdims=True)
        var = t.var(axis=1, keepdims=True)
        out[j] = ((t - mu) / np.sqrt(var + 1e-6)).astype(np.float32)
    return out


def block_stream(name, images):
    """Un-normalised fp32 residual-stream tokens [len(images), N, D] for the pre-LayerNorm block:
    N(0,1) values with a per-token scale in [0.5, 3] and shift in [-1, 1]."""
    d = BLOCKS[name]
    N, D = d["N"], d["D"]
    out = np.empty((len(images), N, D), np.float32)
    for j, i in enumerate(images):
        rng = np.random.default_rng([seed_for(d["cfg"]), 3000, int(i)])
        t = rng.standard_normal((N, D))
        out[j] = (t * rng.uniform(0.5, 3.0, (N, 1)) + rng.uniform(-1.0, 1.0, (N, 1))).astype(np.float32)
    return out


def block_ln_params(name):
    """LayerNorm parameters of the pre-LayerNorm block: gamma ~ 1 + N(0, 0.1), beta ~ N(0, 0.05)."""
    d = BLOCKS[name]
    rng = np.random.default_rng([seed_for(d["cfg"]), 4000])
    D = d["D"]
    return dict(g1=(1 + 0.1 * rng.standard_normal(D)).astype(np.float32),
                b1=(0.05 * rng.standard_normal(D)).astype(np.float32),
                g2=(1 + 0.1 * rng.standard_normal(D)).astype(np.float32),
                b2=(0.05 * rng.standard_normal(D)).astype(np.float32), eps=np.float32(1e-6))


def steps_key(name, sharp, bits_w, bits_a):
    return "%s/%s/w%da%d" % (name, "sharp" if sharp else "stated", bits_w, bits_a)


def block_steps(name, sharp=False, bits_w=4, bits_a=4):
    """Per-tensor activation steps (fp32) of a workload, read from the recorded table.

    The table is written by ``oracle/calibrate_steps.py`` (absmax calibration over two images
    run through the CPU oracle); here the numbers are plain inputs.
    """
    with open(STEPS_FILE) as f:
        table = json.load(f)
    rec = table[steps_key(name, sharp, bits_w, bits_a)]
    return {k: np.float32(float.fromhex(v)) for k, v in rec.items()}
