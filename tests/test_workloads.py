"""Input-generator checks: bf16 rounding against a library conversion, ragged bookkeeping, determinism."""
import numpy as np
import torch

from paper_2402_05099_amd import workloads as wl


def test_bf16_rne_matches_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65280.0, 1e-30], np.float32)])
    mine = wl.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(mine, ref)
    assert np.array_equal(wl.bf16_bits_to_f32(mine), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_lengths_offsets_and_determinism():
    w = wl.scaled_down(4)
    assert w.lengths.min() >= 1 and w.lengths.max() <= 150
    assert w.offsets[0] == 0 and np.array_equal(w.offsets[1:], np.cumsum(w.lengths)[:-1])
    assert w.Ks.shape == (int(w.lengths.sum()), w.Hkv, w.D)
    w2 = wl.scaled_down(4)
    assert np.array_equal(w.Q, w2.Q) and np.array_equal(w.Ks, w2.Ks) and np.array_equal(w.lengths, w2.lengths)


def test_thread_count_does_not_change_values():
    a = wl.normal_bf16(5, 3, (3, (1 << 22) + 17), threads=1)
    b = wl.normal_bf16(5, 3, (3, (1 << 22) + 17), threads=4)
    assert np.array_equal(a, b)
    f = wl.bf16_bits_to_f32(a)
    assert abs(float(f.mean())) < 2e-3 and abs(float(f.std()) - 1.0) < 2e-3


def test_config_shapes():
    w = wl.config(1)
    assert (w.B, w.Hq, w.Hkv, w.D) == (4, 4, 4, 64) and w.levels[0].K.shape == (128, 4, 64)
    assert np.all(w.lengths == 16) and abs(w.scale - 0.125) < 1e-15
    t = wl.scaled_down(5)
    assert t.levels[1].Gn == 4 and t.kv_rows_of(25) == [(0, 0, 200), (1, 77, 154)]


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU: asking for more exits with a message that says so (before anything touches a GPU)."""
    import subprocess
    import sys
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
