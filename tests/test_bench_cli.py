"""Host-side behaviour of bench.py and of the synthetic input recipes (no GPU needed)."""
import os
import subprocess
import sys

import numpy as np

from paper_2505_24133_amd import synth


def test_bench_refuses_more_than_one_gpu(repo_root):
    r = subprocess.run([sys.executable, os.path.join(repo_root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_workload_shapes_follow_the_configuration():
    """N = budget + 128 buffered tokens, alpha = 8, d = 128; problems = layers x sequences."""
    want = {"cfg1_tiny": (1, 2, 8, 384, 256), "cfg2_llama8b_b1024": (32, 8, 32, 1152, 1024),
            "cfg3_llama8b_b4096": (32, 8, 32, 4224, 4096), "cfg4_qwen14b_b2048_bs16": (48 * 16, 8, 40, 2176, 2048),
            "cfg5_llama8b_b8192_bs4": (32 * 4, 8, 32, 8320, 8192)}
    for name, (P, H, Hq, N, B) in want.items():
        w = synth.CONFIGS[name]
        assert (w.num_problems, w.kv_heads, w.q_heads, w.n_tokens, w.budget) == (P, H, Hq, N, B), name
        assert w.alpha == 8 and w.head_dim == 128 and w.n_tokens - w.budget == 128
        assert w.n_cand == N - 8 and w.k_sel == B - 8 and w.group == Hq // H


def test_batches_are_seeded_and_bf16_exact():
    w = synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], num_problems=2)
    q1, k1, v1 = synth.make_batch(w)
    q2, k2, v2 = synth.make_batch(w)
    assert np.array_equal(k1, k2) and np.array_equal(q1, q2) and np.array_equal(v1, v2)
    assert k1.dtype == np.uint16 and k1.shape == (2, 8, 1152, 128) and q1.shape == (2, 32, 8, 128)
    x = np.float32([1.0, -2.5, 3.1415927, 1e-3, 65504.0])
    bits = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(bits)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)              # round to nearest: half an ulp of 8 bits
    assert np.array_equal(synth.f32_to_bf16_bits(back), bits)            # bf16 values are fixed points
    # the copy spans make a sizeable share of rows near-duplicates of an earlier row
    kf = synth.bf16_bits_to_f32(k1[0, 0, :w.n_cand]).astype(np.float64)
    kn = kf / np.linalg.norm(kf, axis=1, keepdims=True)
    S = kn @ kn.T
    np.fill_diagonal(S, 0.0)
    dup = (np.tril(S, -1).max(axis=1) > 0.99).mean()
    assert 0.25 < dup < 0.55
