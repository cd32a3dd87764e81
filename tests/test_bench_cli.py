"""bench.py on the CPU: what it counts as a step's work, and that it refuses more than one GPU."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_flops_of_the_language_step_by_hand():
    """The numerator of the metric.  By hand for the language stage (4 layers, hidden 4096, 32 x 128 heads, FFN 11008
    SwiGLU, T 4096, causal): weights per layer 4 * 4096^2 + 3 * 4096 * 11008 = 202,375,168; a GEMM pass over them for
    4096 tokens is 2 * 4096 * 202,375,168 = 1.65786e12 flop; the attention forward 4 * 128 * 32 * 4096^2 / 2 =
    1.37439e11.  F = 4 * (1.65786e12 + 1.37439e11) = 7.18119e12, B = 4 * (1.65786e12 + 2 * 1.37439e11) = 7.73095e12,
    W = 4 * 1.65786e12 = 6.63143e12; eight microbatches: 1.72349e14."""
    import bench
    import stage_inputs as SI
    fl = bench.task_flops(SI.LANGUAGE, np.array([0, 4096]))
    assert abs(fl["F"] / 7.18119e12 - 1) < 1e-5
    assert abs(fl["B"] / 7.73095e12 - 1) < 1e-5
    assert abs(fl["W"] / 6.63143e12 - 1) < 1e-5
    assert abs(8 * (fl["F"] + fl["B"] + fl["W"]) / 1.72349e14 - 1) < 1e-5


def test_flops_of_a_packed_bidirectional_microbatch():
    """Two segments, no causal mask: attention pairs are the sum of the squared segment lengths, not T^2."""
    import bench
    import stage_inputs as SI
    shape = SI.TINY.replace(causal=False, n_layers=1)
    cu = np.array([0, 3, 10])
    fl = bench.task_flops(shape, cu)
    P = shape.hidden * (shape.n_q_heads + 2 * shape.n_kv_heads) * shape.head_dim + shape.n_q_heads * shape.head_dim * shape.hidden \
        + 3 * shape.hidden * shape.ffn
    att = 4.0 * shape.head_dim * shape.n_q_heads * (3 * 3 + 7 * 7)
    assert fl["F"] == 2.0 * 10 * P + att and fl["B"] == 2.0 * 10 * P + 2 * att and fl["W"] == 2.0 * 10 * P
