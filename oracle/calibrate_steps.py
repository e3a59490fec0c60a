"""Write paper_2504_18547_amd/workload_steps.json: per-tensor activation steps of every workload.

The paper's steps come from a trained low-bit checkpoint (Sec. V-A) that is not available, so
they are calibrated here instead: step = max|t| / qmax over the fp32 tensor t that feeds each
quantizer, measured while a few images run through the CPU oracle stage by stage (an all-zero
tensor gets step 1).  Only oracle/ and the seeded input generators are used.  The resulting
numbers are plain inputs to both the oracle and the GPU library.

Run:  python -m oracle.calibrate_steps            (every workload)
      python -m oracle.calibrate_steps NAME ...   (only these workloads; the other entries are kept)
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from oracle import vqo  # noqa: E402
from paper_2504_18547_amd import workloads as wl  # noqa: E402

VARIANTS = [
    # (workload, images used, [(bits_w, bits_a)])
    ("tiny_attn", [0, 1, 2], [(4, 4), (8, 8), (2, 4), (3, 4)]),
    ("tiny_block", [0, 1], [(4, 4), (8, 8), (2, 4), (3, 4)]),
    ("tiny_long", [0, 1], [(4, 4), (8, 8)]),
    ("deit_s_table1", [0], [(4, 4), (3, 4)]),
    ("vit_s_attn", [0, 1], [(4, 4)]),
    ("vit_b_block_b128", [0, 1], [(4, 4)]),
    ("vit_b_block", [0, 1], [(4, 4), (3, 4), (2, 4), (8, 8)]),
    ("vit_l_577_block", [0], [(4, 4), (8, 8)]),
]


def _absmax_step(t, bits):
    qmax = 2 ** (bits - 1) - 1
    m = np.float32(np.abs(t).max())
    return np.float32(1.0) if m == 0 else np.float32(m / np.float32(qmax))


def quantize_weights(w_fp, bits_w):
    out = {}
    for name in ("qkv", "proj", "fc1", "fc2"):
        if "w_" + name not in w_fp:
            continue
        s = vqo.weight_steps(w_fp["w_" + name], bits_w)
        out["w_" + name] = vqo.quantize(w_fp["w_" + name], s, bits_w, per_row=True)
        out["sw_" + name] = s
        out["b_" + name] = w_fp["b_" + name]
    return out


def calibrate(name, images, sharp, bits_w, bits_a):
    d = wl.block_dims(name)
    D, H, N, hidden = d["D"], d["H"], d["N"], d["hidden"]
    dh, B = D // H, len(images)
    bits_p = bits_a
    pmax = 2 ** bits_p - 1
    wts = quantize_weights(wl.block_weights(name, sharp=sharp), bits_w)
    x = wl.block_tokens(name, images).reshape(B * N, D)
    st = {"scale": np.float32(1.0 / np.sqrt(np.float32(dh)))}
    st["s_x"] = _absmax_step(x, bits_a)
    xq = vqo.quantize(x, st["s_x"], bits_a)
    y = vqo.linear(xq, st["s_x"], wts["w_qkv"], wts["sw_qkv"], bias=wts["b_qkv"], want_acc=False)["y"]
    y5 = y.reshape(B, N, 3, H, dh).transpose(2, 0, 3, 1, 4)
    qkv = []
    for i, key in enumerate(("s_q", "s_k", "s_v")):
        st[key] = _absmax_step(y5[i], bits_a)
        qkv.append(vqo.quantize(np.ascontiguousarray(y5[i]).reshape(-1, dh), st[key], bits_a).reshape(B, H, N, dh))
    p = vqo.matmul_qk(qkv[0], qkv[1], st["s_q"], st["s_k"], st["scale"], bits_p, want_s=False)["p"]
    o = vqo.matmul_pv(p, qkv[2], np.float32(1.0) / np.float32(pmax), st["s_v"])["o"]
    st["s_o"] = _absmax_step(o, bits_a)
    oq = vqo.quantize(o, st["s_o"], bits_a)
    info = dict(p_nonzero=float((p > 0).mean()), p_max=int(p.max()))
    if hidden:
        y2 = vqo.linear(oq, st["s_o"], wts["w_proj"], wts["sw_proj"], bias=wts["b_proj"], want_acc=False)["y"]
        st["s_x2"] = _absmax_step(y2, bits_a)
        x2 = vqo.quantize(y2, st["s_x2"], bits_a)
        g = vqo.linear(x2, st["s_x2"], wts["w_fc1"], wts["sw_fc1"], bias=wts["b_fc1"], act=1, want_acc=False)["y"]
        st["s_h"] = _absmax_step(g, bits_a)
    return st, info


def main():
    table = {}
    only = set(sys.argv[1:])
    if only and os.path.exists(wl.STEPS_FILE):
        with open(wl.STEPS_FILE) as f:
            table = json.load(f)
    for name, images, combos in VARIANTS:
        if only and name not in only:
            continue
        for bits_w, bits_a in combos:
            for sharp in (False, True):
                st, info = calibrate(name, images, sharp, bits_w, bits_a)
                key = wl.steps_key(name, sharp, bits_w, bits_a)
                table[key] = {k: float(v).hex() for k, v in st.items()}
                print(key, {k: float(v) for k, v in st.items()}, info, flush=True)
    with open(wl.STEPS_FILE, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", wl.STEPS_FILE)


if __name__ == "__main__":
    main()
