"""Host-side checks of bench.py's contract that need no GPU: the one-GPU rule, the algorithmic FLOP count behind the
model-FLOPs figure, and the traffic figure taken from the committed counter summary."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench                      # noqa: E402
import dipaco_inputs as gen       # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus 1" in r.stderr


def test_step_flops_are_the_algorithmic_count():
    """Config 2: 2 x (parameters in matrices) x tokens for each of forward, input gradient and weight gradient, plus the
    causal attention products at half a square (forward 2, backward 4); nothing recomputed is counted."""
    cfg = gen.CONFIGS[2]
    B, S = cfg["batch"], cfg["seq"]
    fwd, dx, dw = bench.step_gemm_shapes(cfg, B, S)
    d, A, F, V = cfg["d_model"], cfg["n_heads"] * cfg["d_head"], cfg["d_mlp"], cfg["vocab"]
    matrix_params = 12 * (d * 3 * A + A * d + d * F + F * d) + d * V
    one_pass = 2.0 * matrix_params * B * S
    for launches in (fwd, dx, dw):
        assert len(launches) == 49
        assert sum(2.0 * m * n * k for m, n, k in launches) == one_pass
    a_fwd, a_bwd = bench.attention_flops(cfg, B, S)
    assert a_fwd == 12 * B * cfg["n_heads"] * 2 * (2 * S * S * cfg["d_head"]) / 2 and a_bwd == 2 * a_fwd
    total = 3 * one_pass + a_fwd + a_bwd
    assert abs(total / 1e12 - 30.53) < 0.01


def test_traffic_figure_comes_from_the_committed_summary():
    t = bench.fwd_gemm_traffic_bytes()
    assert t is not None and 3.66e8 <= t <= 1.0e9            # at least the algorithmic 366 MB per launch
    with open(bench.TRAFFIC_PROFILE) as f:
        last = [line for line in f if line.strip()][-1]
    assert last.split()[0] == "TRAFFIC_BYTES_PER_LAUNCH_FWD_GEMM" and float(last.split()[1]) == t
