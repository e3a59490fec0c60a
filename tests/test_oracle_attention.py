"""Pins for the oracle's attention matmuls and the whole-block chain (CPU only)."""
import numpy as np


def _qkv(rng, B=2, H=3, N=11, dh=64, bits=4):
    lo, hi = -(2 ** (bits - 1)), 2 ** (bits - 1) - 1
    return [rng.integers(lo, hi + 1, (B, H, N, dh)).astype(np.int8) for _ in range(3)]


def test_qk_scores_vs_numpy_and_rows_vs_softmax_row(vqo):
    rng = np.random.default_rng(21)
    q, k, _ = _qkv(rng)
    out = vqo.matmul_qk(q, k, 0.21, 0.17, 0.125, 4)
    ref = np.einsum("bhid,bhjd->bhij", q.astype(np.int64), k.astype(np.int64))
    assert np.array_equal(out["s_acc"], ref)
    a = vqo.alpha(0.21, 0.17, 0.125)
    for (b, h, i) in ((0, 0, 0), (1, 2, 10), (0, 1, 5)):
        p, _, _ = vqo.softmax_row(ref[b, h, i].astype(np.int32), a, 15)
        assert np.array_equal(out["p"][b, h, i], p)
    assert out["p"].max() > 3       # not a degenerate all-zero test
    assert np.abs(ref).max() <= 64 * 8 * 8


def test_pv_vs_numpy_and_output_layout(vqo):
    rng = np.random.default_rng(22)
    B, H, N, dh = 2, 3, 9, 64
    _, _, v = _qkv(rng, B, H, N, dh)
    p = rng.integers(0, 16, (B, H, N, N)).astype(np.uint8)
    s_p, s_v, s_o = np.float32(1 / 15), np.float32(0.3), np.float32(0.9)
    out = vqo.matmul_pv(p, v, s_p, s_v, s_o=s_o, bits_o=4)
    ref = np.einsum("bhij,bhjd->bhid", p.astype(np.int64), v.astype(np.int64))
    assert np.array_equal(out["o_acc"], ref)
    # heads are concatenated along the channel axis of a [B*N, H*dh] matrix
    want = ref.transpose(0, 2, 1, 3).reshape(B * N, H * dh).astype(np.float32) * (s_p * s_v)
    assert np.array_equal(out["o"], want)
    assert np.array_equal(out["oq"], vqo.quantize(out["o"], s_o, 4))
    assert len(np.unique(out["oq"])) > 4


def test_one_hot_attention_copies_value_rows(vqo):
    rng = np.random.default_rng(23)
    B, H, N, dh = 1, 2, 7, 64
    _, _, v = _qkv(rng, B, H, N, dh)
    perm = rng.permutation(N)
    p = np.zeros((B, H, N, N), np.uint8)
    p[:, :, np.arange(N), perm] = 15
    out = vqo.matmul_pv(p, v, np.float32(1 / 15), np.float32(1.0))
    assert np.array_equal(out["o_acc"], 15 * v[:, :, perm, :].astype(np.int32))
    np.testing.assert_allclose(out["o"].reshape(N, H, dh).transpose(1, 0, 2),
                               v[0][:, perm, :].astype(np.float32), rtol=2e-7)


def _tiny_block(vqo, rng, D=128, H=2, N=13, hidden=256, B=2):
    dims = dict(D=D, H=H, N=N, hidden=hidden)
    wts = {}
    for name, shape in (("qkv", (3 * D, D)), ("proj", (D, D)), ("fc1", (hidden, D)), ("fc2", (D, hidden))):
        if hidden == 0 and name.startswith("fc"):
            continue
        w = (rng.standard_normal(shape) * (0.08 if name == "qkv" else 0.02)).astype(np.float32)
        s = vqo.weight_steps(w, 4)
        wts["w_" + name] = vqo.quantize(w, s, 4, per_row=True)
        wts["sw_" + name] = s
        wts["b_" + name] = (rng.standard_normal(shape[0]) * 0.01).astype(np.float32)
    x = rng.standard_normal((B * N, D)).astype(np.float32)
    steps = dict(s_x=np.float32(0.5), s_q=np.float32(0.35), s_k=np.float32(0.33), s_v=np.float32(0.1),
                 s_o=np.float32(0.03), s_x2=np.float32(0.012), s_h=np.float32(0.01), scale=np.float32(0.125))
    xq = vqo.quantize(x, steps["s_x"], 4)
    return dims, wts, steps, xq


def test_block_chain_equals_stage_by_stage_composition(vqo):
    """The chain's plumbing (channel -> (q/k/v, head, d) mapping, head concatenation, which step
    feeds which stage) rebuilt here with numpy reshapes around the separately pinned stages."""
    rng = np.random.default_rng(24)
    for hidden in (0, 256):
        dims, wts, st, xq = _tiny_block(vqo, rng, hidden=hidden)
        D, H, N, B = dims["D"], dims["H"], dims["N"], 2
        dh = D // H
        out = vqo.attention_block(xq, B, dims, wts, st, dump_p=True)

        y = vqo.linear(xq, st["s_x"], wts["w_qkv"], wts["sw_qkv"], bias=wts["b_qkv"])["y"]
        y5 = y.reshape(B, N, 3, H, dh).transpose(2, 0, 3, 1, 4)            # [3][B][H][N][dh]
        q = vqo.quantize(y5[0].reshape(-1, dh), st["s_q"], 4).reshape(B, H, N, dh)
        k = vqo.quantize(y5[1].reshape(-1, dh), st["s_k"], 4).reshape(B, H, N, dh)
        v = vqo.quantize(y5[2].reshape(-1, dh), st["s_v"], 4).reshape(B, H, N, dh)
        assert np.array_equal(out["q"], q) and np.array_equal(out["k"], k) and np.array_equal(out["v"], v)
        p = vqo.matmul_qk(q, k, st["s_q"], st["s_k"], st["scale"], 4)["p"]
        assert np.array_equal(out["p"], p)
        assert p.max() >= 4 and (p > 0).mean() > 0.05                      # not degenerate
        o = vqo.matmul_pv(p, v, np.float32(1.0) / np.float32(15), st["s_v"], s_o=st["s_o"])["oq"]
        assert np.array_equal(out["o"], o)
        assert len(np.unique(o)) > 4
        if hidden == 0:
            yy = vqo.linear(o, st["s_o"], wts["w_proj"], wts["sw_proj"], bias=wts["b_proj"])["y"]
            assert np.array_equal(out["y"], yy)
        else:
            pr = vqo.linear(o, st["s_o"], wts["w_proj"], wts["sw_proj"], bias=wts["b_proj"],
                            s_y=st["s_x2"], bits_y=4)
            assert np.array_equal(out["x2"], pr["yq"]) and np.array_equal(out["y_attn"], pr["y"])
            f1 = vqo.linear(pr["yq"], st["s_x2"], wts["w_fc1"], wts["sw_fc1"], bias=wts["b_fc1"], act=1,
                            s_y=st["s_h"], bits_y=4)
            assert np.array_equal(out["h"], f1["yq"])
            assert len(np.unique(f1["yq"])) > 4
            f2 = vqo.linear(f1["yq"], st["s_h"], wts["w_fc2"], wts["sw_fc2"], bias=wts["b_fc2"])
            assert np.array_equal(out["y"], f2["y"])


def test_images_are_independent_and_threads_do_not_matter(vqo):
    rng = np.random.default_rng(25)
    dims, wts, st, xq = _tiny_block(vqo, rng, hidden=256, B=3)
    N = dims["N"]
    full = vqo.attention_block(xq, 3, dims, wts, st, threads=3)
    one = vqo.attention_block(xq[N:2 * N], 1, dims, wts, st, threads=1)
    assert np.array_equal(full["y"][N:2 * N], one["y"])
    assert np.array_equal(full["h"][N:2 * N], one["h"])
