"""CPU oracle for the ReKV hot path (test infrastructure, not the product).

A plain, slow, fp64 numpy statement of what the method computes, written from
the paper's method section.  Only tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it.  It shares no code with the HIP path and
imports nothing from it.  Every function here is pinned by the CPU tests
(brute force on tiny inputs, library special cases, closed forms, invariants);
none is "parity unpinned".

Layouts: token-major.  Q is [tokens, Hq, D]; K and V are [tokens, Hkv, D].
Query head h reads KV head h // G with G = Hq / Hkv (contiguous groups).

Readings where the paper is silent are listed next to the function they touch.
"""
from __future__ import annotations

import math

import numpy as np


def _f64(x):
    return np.asarray(x, dtype=np.float64)


def softmax_attention(q, k, v, visible, scale):
    """Attn(Q, K, V) for one head: softmax(scale * Q K^T restricted to `visible`) V.

    The paper writes Attn(.) without defining it (Eq. 1, Eq. 3); this is standard
    scaled dot-product attention.  q [m, D], k/v [n, D], visible [m, n] bool with
    at least one True per row.  Returns (O [m, D], P [m, n]).
    """
    z = scale * (_f64(q) @ _f64(k).T)
    z = np.where(visible, z, -np.inf)
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    p = e / e.sum(axis=1, keepdims=True)
    return p @ _f64(v), p


def encode_chunks(q, k_cache, v_cache, first_token, l_x, n_chunks, l_l, scale=None,
                  return_probs=False):
    """Sliding-window chunk attention, Eq. 1 (video stream encoding).

    Chunk c holds tokens [t0, t0 + l_x), t0 = first_token + c * l_x.  Its past is
    P = tokens [0, t0); the local window is L = the last min(l_l, t0) tokens of P
    (when the stream is younger than the window, L is all of P).  Every token of
    the chunk gets the same L (the window is anchored at the chunk start, as Eq. 1
    is written) and sees the chunk's own tokens causally.

    q [n_chunks * l_x, Hq, D] holds the chunks' queries; k_cache / v_cache
    [>= first_token + n_chunks * l_x, Hkv, D] hold the stream's keys / values
    including the chunks' own.  Returns O [n_chunks * l_x, Hq, D] (and the list of
    per-(chunk, head) probability matrices if asked).
    """
    q, k_cache, v_cache = _f64(q), _f64(k_cache), _f64(v_cache)
    n_q_heads, d = q.shape[1], q.shape[2]
    group = n_q_heads // k_cache.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    out = np.empty_like(q)
    probs = []
    for c in range(n_chunks):
        t0 = first_token + c * l_x
        w0 = max(0, t0 - l_l)
        n_win = t0 - w0
        # key column j of the slice is stream token w0 + j; query row i is token t0 + i
        visible = np.ones((l_x, n_win + l_x), dtype=bool)
        visible[:, n_win:] = np.tril(np.ones((l_x, l_x), dtype=bool))
        for h in range(n_q_heads):
            g = h // group
            o, p = softmax_attention(q[c * l_x:(c + 1) * l_x, h], k_cache[w0:t0 + l_x, g],
                                     v_cache[w0:t0 + l_x, g], visible, scale)
            out[c * l_x:(c + 1) * l_x, h] = o
            if return_probs:
                probs.append(p)
    return (out, probs) if return_probs else out


def frame_keys(k, n_frames, tokens_per_frame):
    """Representative frame vector: the mean of the frame's N_f key vectors, the
    KV heads concatenated into one vector of D' = Hkv * D (internal retrieval).

    k [>= n_frames * N_f, Hkv, D] -> [n_frames, D'].
    """
    k = _f64(k)[: n_frames * tokens_per_frame]
    d_prime = k.shape[1] * k.shape[2]
    return k.reshape(n_frames, tokens_per_frame, d_prime).sum(axis=1) / tokens_per_frame


def question_vector(q_question, n_kv_heads):
    """Question vector: the mean of the N_q query vectors, heads concatenated.

    Under grouped-query attention the concatenated queries have Hq * D entries but
    the frame vectors Hkv * D.  Reading taken: average the G query heads that share
    a KV head, which gives a vector of D' = Hkv * D.  (Repeating every key head G
    times instead scales all scores by one positive constant, so it ranks frames
    identically; `test_oracle_pins` checks that.)

    q_question [N_q, Hq, D] -> [D'].
    """
    q = _f64(q_question)
    n_q, n_q_heads, d = q.shape
    group = n_q_heads // n_kv_heads
    per_head = q.sum(axis=0) / n_q                      # [Hq, D]
    return (per_head.reshape(n_kv_heads, group, d).sum(axis=1) / group).reshape(-1)


def cosine_scores(frame_vecs, q_vec, tau=1.0):
    """Eq. 2: Sim(v, q) = v.q / (tau |v| |q|), tau = 1 for internal retrieval.
    One cosine over the whole concatenated vector.  A zero-norm vector scores 0.

    frame_vecs [F, D'], q_vec [D'] -> [F].
    """
    v, qv = _f64(frame_vecs), _f64(q_vec)
    dots = v @ qv
    den = tau * np.sqrt((v * v).sum(axis=1)) * math.sqrt(float(qv @ qv))
    return np.where(den > 0, dots / np.where(den > 0, den, 1.0), 0.0)


def topk_frames(scores, k):
    """The r most similar frames.  Ties go to the lower frame index; the selected
    frames are reported in ascending (temporal) order.  If k exceeds the number of
    frames, all frames are selected.  Returns an int64 array of min(k, F) indices.
    """
    s = _f64(scores)
    order = sorted(range(len(s)), key=lambda f: (-s[f], f))
    return np.array(sorted(order[: min(k, len(s))]), dtype=np.int64)


def gather_kv(k, v, frames, tokens_per_frame):
    """Retrieved KV R: the selected frames' key and value blocks, in the order given."""
    rows = np.concatenate([np.arange(f * tokens_per_frame, (f + 1) * tokens_per_frame)
                           for f in frames]) if len(frames) else np.zeros(0, dtype=np.int64)
    return np.asarray(k)[rows], np.asarray(v)[rows]


def apply_rope(x, positions, base=10000.0, layout="half"):
    """Rotary position embedding (the paper's positional-encoding paragraph cites RoFormer):
    every head vector is split into D/2 pairs; pair i is rotated by the angle
    position * theta_i, theta_i = base^(-2i/D):
        a' = a cos - b sin,   b' = a sin + b cos.
    layout "interleaved" pairs dims (2i, 2i+1) as RoFormer writes it; "half" pairs dims
    (i, i + D/2), the arrangement of the decoder family the paper runs on.  Positions may be
    any integers (negative ones rotate back).

    x [T, H, D], positions [T] -> [T, H, D] fp64.
    """
    x = _f64(x)
    t, _, d = x.shape
    half = d // 2
    theta = np.array([base ** (-2.0 * i / d) for i in range(half)])
    ang = np.asarray(positions, dtype=np.float64).reshape(t, 1, 1) * theta.reshape(1, 1, half)
    c, s_ = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    if layout == "interleaved":
        a, b = x[..., 0::2], x[..., 1::2]
        out[..., 0::2] = a * c - b * s_
        out[..., 1::2] = a * s_ + b * c
    elif layout == "half":
        a, b = x[..., :half], x[..., half:]
        out[..., :half] = a * c - b * s_
        out[..., half:] = a * s_ + b * c
    else:
        raise ValueError(layout)
    return out


def gather_kv_rope(k, v, frames, tokens_per_frame, mode="consecutive", pos_offset=0,
                   src_rotated=False, src_pos_offset=0, base=10000.0, layout="half"):
    """Retrieved KV with the paper's position policy for question answering: the original
    positions of the retrieved tokens are dropped and the tokens are treated as regular
    consecutive tokens (mode "consecutive": gathered token j gets position pos_offset + j);
    the static variant gives every retrieved token the same position (mode "static":
    pos_offset).  Values carry no position.

    The cache may hold keys without positions (src_rotated False) or keys already rotated
    at their stream position src_pos_offset + token index (True); rotations compose, so the
    latter are turned by the difference of the two positions.
    Returns (K' [len(frames) * N_f, Hkv, D] fp64, V likewise)."""
    rk, rv = gather_kv(k, v, frames, tokens_per_frame)
    n = rk.shape[0]
    new_pos = np.full(n, pos_offset, dtype=np.int64)
    if mode == "consecutive":
        new_pos = new_pos + np.arange(n)
    elif mode != "static":
        raise ValueError(mode)
    old_pos = np.zeros(n, dtype=np.int64)
    if src_rotated:
        old_pos = src_pos_offset + np.concatenate(
            [np.arange(int(f) * tokens_per_frame, (int(f) + 1) * tokens_per_frame) for f in frames]
        ).astype(np.int64) if len(frames) else old_pos
    return apply_rope(rk, new_pos - old_pos, base, layout), _f64(rv)


def qa_attention(q, k_ret, v_ret, k_self, v_self, scale=None, return_probs=False):
    """Eq. 3 for X = the question tokens: every question token attends to all of the
    retrieved KV R and, causally, to the question tokens up to itself.  The local
    window is not part of this context.

    q [N_q, Hq, D], k_ret / v_ret [n_ret, Hkv, D], k_self / v_self [N_q, Hkv, D]
    -> O [N_q, Hq, D].
    """
    q = _f64(q)
    n_q, n_q_heads, d = q.shape
    n_ret = np.asarray(k_ret).shape[0]
    keys = np.concatenate([_f64(k_ret), _f64(k_self)])
    vals = np.concatenate([_f64(v_ret), _f64(v_self)])
    group = n_q_heads // keys.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    visible = np.ones((n_q, n_ret + n_q), dtype=bool)
    visible[:, n_ret:] = np.tril(np.ones((n_q, n_q), dtype=bool))
    out = np.empty_like(q)
    probs = []
    for h in range(n_q_heads):
        o, p = softmax_attention(q[:, h], keys[:, h // group], vals[:, h // group],
                                 visible, scale)
        out[:, h] = o
        probs.append(p)
    return (out, probs) if return_probs else out


def decode_attention(q_new, k_ret, v_ret, k_text, v_text, scale=None):
    """Eq. 3 for X = the token(s) being decoded: the context is the retrieved video KV
    followed by the text KV so far (question, generated tokens, and the new tokens'
    own keys and values, which are the last n_new rows of k_text / v_text).  New token
    i attends to all of R and to the text tokens up to and including itself, i.e. to
    text positions <= n_text - n_new + i.

    q_new [n_new, Hq, D], k_ret / v_ret [n_ret, Hkv, D], k_text / v_text [n_text, Hkv, D]
    with n_text >= n_new -> O [n_new, Hq, D].
    """
    q = _f64(q_new)
    n_new, n_q_heads, d = q.shape
    n_ret = np.asarray(k_ret).shape[0]
    n_text = np.asarray(k_text).shape[0]
    if n_text < n_new:
        raise ValueError("the text KV must already hold the new tokens' own rows")
    keys = np.concatenate([_f64(k_ret), _f64(k_text)])
    vals = np.concatenate([_f64(v_ret), _f64(v_text)])
    group = n_q_heads // keys.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    visible = np.ones((n_new, n_ret + n_text), dtype=bool)
    for i in range(n_new):
        visible[i, n_ret + (n_text - n_new + i) + 1:] = False
    out = np.empty_like(q)
    for h in range(n_q_heads):
        out[:, h], _ = softmax_attention(q[:, h], keys[:, h // group], vals[:, h // group],
                                         visible, scale)
    return out


def retrieve(frame_vecs, q_question, n_kv_heads, k, n_visible=None):
    """Internal retrieval for one question: pooled question vector, Eq. 2 scores over
    the frames seen before the question was asked (the question's timestamp cuts off
    later frames), top-k.  Returns (indices ascending, scores [n_visible])."""
    fv = _f64(frame_vecs)
    fv = fv if n_visible is None else fv[:n_visible]
    s = cosine_scores(fv, question_vector(q_question, n_kv_heads))
    return topk_frames(s, k), s


def retrieve_external(frame_emb, q_emb, k, tau=1.0):
    """External retrieval for one question: Eq. 2 with its temperature on embeddings that
    a CLIP-like encoder pair produced elsewhere, then the same top-k rule.
    frame_emb [F, D], q_emb [D].  Returns (indices ascending, scores [F])."""
    s = cosine_scores(frame_emb, q_emb, tau)
    return topk_frames(s, k), s


def block_vectors(frame_vecs, b):
    """Block-level retrieval: b consecutive frames form a block whose vector is the
    average of their frame vectors.  The paper does not say what happens when b does
    not divide the number of frames; here the last block holds the remaining frames and
    averages over those.  frame_vecs [F, D'] -> [ceil(F / b), D']."""
    fv = _f64(frame_vecs)
    n_blocks = -(-fv.shape[0] // b)
    return np.stack([fv[j * b:(j + 1) * b].mean(axis=0) for j in range(n_blocks)])


def expand_blocks(blocks, b, n_frames):
    """The frames of the given blocks, in the order of the blocks: block j holds frames
    j*b .. min((j+1)*b, n_frames) - 1."""
    return np.array([f for j in blocks for f in range(int(j) * b, min((int(j) + 1) * b, n_frames))],
                    dtype=np.int64)


def retrieve_blocks(frame_vecs, q_question, n_kv_heads, r, b):
    """Block-level internal retrieval: Eq. 2 between the pooled question vector and the
    block vectors, the ceil(r / b) most similar blocks (ties to the lower index, reported
    ascending), and all of their frames as the retrieved set (so up to ceil(r/b)*b >= r
    frames).  Returns (frame indices ascending, block indices ascending, block scores)."""
    bv = block_vectors(frame_vecs, b)
    s = cosine_scores(bv, question_vector(q_question, n_kv_heads))
    blocks = topk_frames(s, -(-r // b))
    return expand_blocks(blocks, b, np.asarray(frame_vecs).shape[0]), blocks, s


def kv_cache_bytes(n_layers, n_frames, tokens_per_frame, n_kv_heads, head_dim,
                   bytes_per_value=2):
    """KV-cache size formula of the appendix: keys and values, every layer, every
    frame's tokens, every KV head and dimension."""
    return 2 * n_layers * n_frames * tokens_per_frame * n_kv_heads * head_dim * bytes_per_value
