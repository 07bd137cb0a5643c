"""Host logic of bench.py (no GPU): the algorithmic bytes behind the roofline figures, and the one-GPU guard."""
import os
import subprocess
import sys

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    sys.path.insert(0, ROOT)
    import bench
    return bench


def test_algorithmic_bytes_of_a_forward_are_the_weights_once_plus_the_cache():
    """Hand count for the 70B / 7B shapes: per layer the QKV, O, gate, up and down matrices in bf16, once per forward
    whatever the number of rows, plus the LM head; the K / V of every cached position read once (2 * kv heads * head
    dim * 2 bytes per layer and token), the new rows written, fp32 logits written.  (The embedding is a gather of m
    rows and the gains are vectors: not counted.)"""
    bench = _bench()
    cfg = synth.config("70b_7b")
    t, d = cfg.target, cfg.draft
    per_layer_t = 8192 * (64 + 2 * 8) * 128 + 8192 * 8192 + 3 * 8192 * 28672
    weights_t = 2 * (80 * per_layer_t + 32000 * 8192)
    assert abs(weights_t - 137.43e9) < 0.01e9
    kv_t = 80 * 2 * 8 * 128 * 2                       # bytes per cached token, all layers
    assert kv_t == 327680
    for n_ctx, m in ((4095, 1), (4095, 7), (0, 1)):
        assert bench.forward_bytes(t, n_ctx, m) == weights_t + (n_ctx + m) * kv_t + m * 32000 * 4
    per_layer_d = 4096 * 3 * 4096 + 4096 * 4096 + 3 * 4096 * 11008
    weights_d = 2 * (32 * per_layer_d + 32000 * 4096)
    assert abs(weights_d - 13.21e9) < 0.01e9
    kv_d = 32 * 2 * 32 * 128 * 2
    assert bench.forward_bytes(d, 4095, 1) == weights_d + 4096 * kv_d + 32000 * 4
    # a PEARL step at gamma 7 moves about 246 GB
    step = bench.forward_bytes(t, 4096, 7) + 7 * bench.forward_bytes(d, 4096, 1)
    assert abs(step - 246.4e9) < 0.3e9


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
