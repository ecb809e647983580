"""Host-side logic of bench.py that needs no GPU: the single-GPU refusal, the algorithmic work
formulas the roofline figures are priced with, and the bounded CPU baseline."""
import subprocess
import sys
import os

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from oracle import rekv_oracle as O  # noqa: E402
from paper_2503_00540_amd import workloads as W  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "single-GPU" in p.stderr


def test_encode_flops_count_visible_pairs():
    """4 * D * Hq FLOP per visible (query, key) pair, pairs counted from the oracle's own
    visibility on a small stream."""
    w = W.C1.scaled(n_frames=7, tokens_per_frame=5, chunk_frames=1, window_frames=3, name="tiny")
    pairs = 0
    for c in range(w.n_frames):
        t0 = c * w.l_x
        n_win = min(w.l_l, t0)
        for i in range(w.l_x):
            pairs += n_win + i + 1
    assert bench.encode_flops(w) == 4.0 * w.head_dim * w.n_q_heads * pairs
    # the C1 figure quoted in the design notes: 2.2518e12 FLOP per layer
    assert abs(bench.encode_flops(W.C1) / 2.2518e12 - 1) < 1e-4


def test_qa_flops():
    w = W.C1
    pairs = w.n_q_tokens * w.top_k * w.tokens_per_frame + w.n_q_tokens * (w.n_q_tokens + 1) // 2
    assert bench.qa_flops(w) == 4.0 * w.head_dim * w.n_q_heads * w.n_questions * pairs


def test_cpu_baseline_is_bounded_and_reports_what_it_sampled():
    out = bench.cpu_baseline(W.C0, seconds_target=0.5)
    assert out["kind"] == "oracle" and out["unit"] == "video tokens/s" and out["value"] > 0
    assert out["cores"] >= 1 and "chunk" in out["sample"]
