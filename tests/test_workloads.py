"""The seeded input generators: deterministic, independent per frame, exact in the
storage type.  No GPU needed."""
import numpy as np
import torch

from paper_2503_00540_amd import workloads as W


def test_frames_are_independent_and_deterministic():
    w = W.C1.scaled(n_frames=8)
    a = W.frames_k(w, 0, 4)
    b = W.frames_k(w, 2, 3)
    np.testing.assert_array_equal(a[2 * w.tokens_per_frame:3 * w.tokens_per_frame], b)
    np.testing.assert_array_equal(W.frames_k(w, 2, 3), b)
    assert np.abs(W.frames_v(w, 2, 3) - b).max() > 0.1
    assert a.shape == (4 * 196, 4, 128) and a.dtype == np.float32


def test_bf16_rounding_is_exact_and_nearest_even():
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    r = W.round_to_bf16(x)
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, t)
    # values are already on the bf16 grid: a second rounding changes nothing
    np.testing.assert_array_equal(W.round_to_bf16(r), r)
    assert W.frames_q(W.C0, 0, 1).dtype == np.float32


def test_statistics_match_the_recipe():
    w = W.C1.scaled(n_frames=16)
    k = W.frames_k(w, 0, 16).astype(np.float64)
    # unit-variance noise around a per-frame offset of sigma 0.5
    per_frame = k.reshape(16, 196, -1)
    assert abs(per_frame.std(axis=1).mean() - 1.0) < 0.02
    assert abs(per_frame.mean(axis=1).std() - 0.5) < 0.06
    qq, qk, qv = W.question_qkv(w, 0)
    assert qq.shape == (32, 28, 128) and qk.shape == (32, 4, 128)
    p = W.planted_frames(w, 0)
    assert len(p) == 3 and len(set(p)) == 3 and p.max() < 16
    assert list(W.planted_frames(W.C0)) == [7]


def test_parity_chunk_sample():
    assert W.parity_chunks(256, 16) == [0, 1, 15, 16, 17, 128, 192, 255]
    assert W.parity_chunks(3, 16) == [0, 1, 2]
