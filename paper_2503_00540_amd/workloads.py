"""Seeded synthetic inputs shaped like the paper's streaming-VideoQA workloads.

This module only draws random numbers and rounds them to the storage type.
It holds none of the method's arithmetic (no attention, no pooling, no
scoring, no selection), so the tests may feed the same arrays to the CPU
oracle and to the HIP path.

Shapes follow the paper's appendix on KV-cache size (a 7B-class decoder has
4 KV heads of dimension 128 and 196 tokens per frame) and its implementation
details (questions of a few dozen tokens, a few dozen retrieved frames).

Every frame of every tensor has its own counter-based (Philox) stream keyed by
(seed, layer, kind, frame), so any frame can be produced without the others.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

_KIND_OFFSETS, _KIND_Q, _KIND_K, _KIND_V = 0, 1, 2, 3
_KIND_QUESTION = 4


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" or "bf16": the storage type of Q/K/V/O
    n_q_heads: int        # Hq
    n_kv_heads: int       # Hkv
    head_dim: int         # D
    n_frames: int         # F
    tokens_per_frame: int  # N_f
    chunk_frames: int     # chunk size l_X in frames
    window_frames: int    # local window l_L in frames
    n_q_tokens: int       # N_q
    top_k: int            # r, retrieved frames
    n_planted: int        # frames each question is planted near
    n_questions: int = 1
    n_layers: int = 1
    kv_on_host: bool = False
    seed: int = 0x5EED0000

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def l_x(self) -> int:
        return self.chunk_frames * self.tokens_per_frame

    @property
    def l_l(self) -> int:
        return self.window_frames * self.tokens_per_frame

    @property
    def n_tokens(self) -> int:
        return self.n_frames * self.tokens_per_frame

    @property
    def d_prime(self) -> int:
        return self.n_kv_heads * self.head_dim

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five configurations of the benchmark definition, in its order.
C0 = Workload("C0-tiny-f32", "f32", 4, 1, 64, 32, 16, 1, 4, 8, 4, 1, seed=0x5EED0000)
C1 = Workload("C1-7B-1layer", "bf16", 28, 4, 128, 256, 196, 1, 16, 32, 16, 3, seed=0x5EED0001)
C2 = Workload("C2-hour-hostKV", "bf16", 28, 4, 128, 3600, 196, 1, 16, 64, 64, 3,
              kv_on_host=True, seed=0x5EED0002)
C3 = Workload("C3-28layers", "bf16", 28, 4, 128, 1024, 196, 4, 32, 48, 32, 3,
              n_layers=28, seed=0x5EED0003)
C4 = Workload("C4-72B-64questions", "bf16", 64, 8, 128, 2048, 144, 1, 16, 32, 32, 3,
              n_questions=64, seed=0x5EED0004)
CONFIGS = {"C0": C0, "C1": C1, "C2": C2, "C3": C3, "C4": C4}

SIGMA_FRAME_OFFSET = 0.5   # per-frame mean offset
SIGMA_QUESTION = 0.3       # noise on the planted question queries


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); returns float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round to the storage type's grid; the result is float32 holding exact values."""
    x = x.astype(np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


def _rng(w: Workload, layer: int, kind: int, index: int) -> np.random.Generator:
    key = [np.uint64(w.seed), np.uint64((layer << 48) | (kind << 40) | index)]
    return np.random.Generator(np.random.Philox(key=key))


def frame_offsets(w: Workload, frame: int, layer: int = 0):
    """Per-frame mean offsets (off_q [Hq,D], off_k [Hkv,D], off_v [Hkv,D]), sigma 0.5."""
    g = _rng(w, layer, _KIND_OFFSETS, frame)
    oq = SIGMA_FRAME_OFFSET * g.standard_normal((w.n_q_heads, w.head_dim))
    ok = SIGMA_FRAME_OFFSET * g.standard_normal((w.n_kv_heads, w.head_dim))
    ov = SIGMA_FRAME_OFFSET * g.standard_normal((w.n_kv_heads, w.head_dim))
    return oq, ok, ov


def _frame_tensor(w: Workload, frame: int, layer: int, kind: int) -> np.ndarray:
    oq, ok, ov = frame_offsets(w, frame, layer)
    off, heads = {_KIND_Q: (oq, w.n_q_heads), _KIND_K: (ok, w.n_kv_heads),
                  _KIND_V: (ov, w.n_kv_heads)}[kind]
    g = _rng(w, layer, kind, frame)
    x = g.standard_normal((w.tokens_per_frame, heads, w.head_dim)) + off[None]
    return to_storage(x, w.dtype)


def frames_q(w: Workload, f0: int, f1: int, layer: int = 0) -> np.ndarray:
    """Queries of frames [f0, f1): [(f1-f0)*N_f, Hq, D], values exact in the storage type."""
    return np.concatenate([_frame_tensor(w, f, layer, _KIND_Q) for f in range(f0, f1)])


def frames_k(w: Workload, f0: int, f1: int, layer: int = 0) -> np.ndarray:
    return np.concatenate([_frame_tensor(w, f, layer, _KIND_K) for f in range(f0, f1)])


def frames_v(w: Workload, f0: int, f1: int, layer: int = 0) -> np.ndarray:
    return np.concatenate([_frame_tensor(w, f, layer, _KIND_V) for f in range(f0, f1)])


def planted_frames(w: Workload, question: int = 0, layer: int = 0,
                   n_visible: int | None = None) -> np.ndarray:
    """The frames a question is planted near (sorted). C0 plants frame 7 by definition."""
    if w.name.startswith("C0"):
        return np.array([7], dtype=np.int64)
    n_visible = w.n_frames if n_visible is None else n_visible
    g = _rng(w, layer, _KIND_QUESTION, 2 * question)
    return np.sort(g.choice(n_visible, size=w.n_planted, replace=False)).astype(np.int64)


def question_qkv(w: Workload, question: int = 0, layer: int = 0,
                 n_visible: int | None = None):
    """Question tokens' (q [N_q,Hq,D], k [N_q,Hkv,D], v [N_q,Hkv,D]).

    Query token t of every head is a noisy copy (sigma 0.3) of the key offset of
    planted frame p[t mod P] for that head's KV group: the offset is the expected
    value of the frame's keys, so the queries sit near that frame's mean key.
    """
    p = planted_frames(w, question, layer, n_visible)
    g = _rng(w, layer, _KIND_QUESTION, 2 * question + 1)
    q = np.empty((w.n_q_tokens, w.n_q_heads, w.head_dim))
    offs = [frame_offsets(w, int(f), layer)[1] for f in p]
    for t in range(w.n_q_tokens):
        ok = offs[t % len(p)]                       # [Hkv, D]
        q[t] = np.repeat(ok, w.group, axis=0)       # head h copies group h // G
    q += SIGMA_QUESTION * g.standard_normal(q.shape)
    k = g.standard_normal((w.n_q_tokens, w.n_kv_heads, w.head_dim))
    v = g.standard_normal((w.n_q_tokens, w.n_kv_heads, w.head_dim))
    return to_storage(q, w.dtype), to_storage(k, w.dtype), to_storage(v, w.dtype)


def parity_chunks(n_chunks: int, window_chunks: int) -> list[int]:
    """Chunks sampled for parity at sizes the oracle cannot run whole: the first two,
    the two around the point where the window fills, three in steady state, the last."""
    cand = [0, 1, window_chunks - 1, window_chunks, window_chunks + 1,
            n_chunks // 2, (3 * n_chunks) // 4, n_chunks - 1]
    return sorted({c for c in cand if 0 <= c < n_chunks})
