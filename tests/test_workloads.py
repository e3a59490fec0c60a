"""Host-side checks of the seeded input generators and the recorded step table (CPU only)."""
import numpy as np

from paper_2504_18547_amd import workloads as wl


def test_recorded_steps_are_reproduced_by_the_calibration_script():
    from oracle import calibrate_steps as cs
    for name, images, combos in cs.VARIANTS[:2]:
        for bits_w, bits_a in combos[:2]:
            for sharp in (False, True):
                st, _ = cs.calibrate(name, images, sharp, bits_w, bits_a)
                rec = wl.block_steps(name, sharp, bits_w, bits_a)
                assert set(st) == set(rec)
                for k in st:
                    assert np.float32(st[k]) == rec[k], (name, sharp, bits_w, bits_a, k)


def test_generators_are_seeded_and_per_image():
    a = wl.block_tokens("tiny_block", [0, 1, 2])
    b = wl.block_tokens("tiny_block", [2])
    assert np.array_equal(a[2], b[0])
    assert a.dtype == np.float32 and a.shape == (3, 50, 128)
    assert abs(float(a.mean())) < 1e-3 and abs(float(a.std()) - 1.0) < 1e-2       # LayerNormed
    w1 = wl.block_weights("tiny_block")
    w2 = wl.block_weights("tiny_block")
    assert all(np.array_equal(w1[k], w2[k]) for k in w1)
    ws = wl.block_weights("vit_s_attn", sharp=True)
    assert abs(float(ws["w_qkv"][:768].std()) - 0.08) < 2e-3
    assert abs(float(ws["w_qkv"][768:].std()) - 0.02) < 1e-3
    c1 = wl.linear_cfg1_inputs()
    assert c1["x"].shape == (197, 384) and c1["w"].shape == (1152, 384) and c1["bias"].shape == (1152,)
    assert abs(float(c1["w"].std()) - 0.02) < 5e-4 and abs(float(c1["bias"].std()) - 0.01) < 1e-3


def test_every_benchmark_workload_has_steps():
    for name, bw, ba in (("vit_s_attn", 4, 4), ("vit_b_block_b128", 4, 4), ("vit_b_block", 4, 4),
                         ("vit_b_block", 3, 4), ("vit_b_block", 2, 4), ("vit_b_block", 8, 8),
                         ("vit_l_577_block", 4, 4), ("vit_l_577_block", 8, 8)):
        for sharp in (False, True):
            st = wl.block_steps(name, sharp, bw, ba)
            assert all(np.isfinite(v) and v > 0 for v in st.values())


def test_bench_refuses_more_than_one_gpu():
    # the path runs on one GPU; asking for more must end with a message, before anything touches a GPU
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
