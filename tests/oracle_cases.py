"""Oracle-side test cases shared by the oracle pins and the GPU parity tests: plain numpy and the
oracle only (no torch, no binding of the HIP library), built from the seeded generators."""
import numpy as np

from oracle import vqo


def quantized_weights(w_fp, bits_w):
    """fp32 weights -> oracle levels / steps / biases (numpy)."""
    out = {}
    for name in ("qkv", "proj", "fc1", "fc2"):
        if "w_" + name not in w_fp:
            continue
        s = vqo.weight_steps(w_fp["w_" + name], bits_w)
        out["w_" + name] = vqo.quantize(w_fp["w_" + name], s, bits_w, per_row=True)
        out["sw_" + name] = s
        out["b_" + name] = w_fp["b_" + name]
    return out


def preln_case(name, sharp, bits_w, bits_a, images):
    """Oracle-side inputs of the pre-LayerNorm block: stream tokens, LayerNorm parameters, weights,
    and steps.  The attention steps are the workload's recorded ones; the two LayerNorm quantizers
    get 3.5/qmax (a unit-variance row clipped at 3.5 sigma), and the GELU output step is calibrated here
    by the oracle (absmax/qmax over the first image)."""
    from paper_2504_18547_amd import workloads as wl
    dims = wl.block_dims(name)
    N, D = dims["N"], dims["D"]
    lo, hi = vqo.qrange(bits_a)
    st = dict(wl.block_steps(name, sharp, bits_w, bits_a))
    st["s_x"] = st["s_x2"] = np.float32(3.5 / hi)
    wts = quantized_weights(wl.block_weights(name, sharp=sharp), bits_w)
    ln = wl.block_ln_params(name)
    x0 = wl.block_stream(name, images[:1]).reshape(N, D)
    first = vqo.vit_block_preln(x0, 1, dims, wts, st, ln, bits_a=bits_a, bits_p=bits_a)
    g = vqo.linear(first["x2"], st["s_x2"], wts["w_fc1"], wts["sw_fc1"], bias=wts["b_fc1"], act=1)["y"]
    st["s_h"] = np.float32(np.abs(g).max() / hi)
    x = wl.block_stream(name, images).reshape(len(images) * N, D)
    return dict(dims=dims, st=st, wts=wts, ln=ln, x=x)
