"""HIP path vs the CPU oracle, element by element, on the same seeded inputs.  Everything
here goes through the C ABI (via the ctypes binding) and needs a real MI355X.

Tolerances (from the benchmark definition): attention outputs max-abs 2e-2 for bf16
inputs and 1e-4 for fp32 inputs; frame vectors and scores 1e-5 (fp32 sums of O(1) values);
top-k indices bit-exact wherever the k-th and (k+1)-th scores differ by more than 1e-3;
gather bit-exact.
"""
import numpy as np
import pytest
import torch

from oracle import rekv_oracle as O
from paper_2503_00540_amd import workloads as W
from paper_2503_00540_amd.rekv import Rekv, RekvError

pytestmark = pytest.mark.gpu
TOL = {"bf16": 2e-2, "f32": 1e-4}
DEV = "cuda:0"


def dev(x, w):
    t = torch.from_numpy(np.ascontiguousarray(x))
    return t.to(torch.bfloat16 if w.dtype == "bf16" else torch.float32).to(DEV)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def check_topk(idx_gpu, scores_oracle, k, gap=1e-3):
    """GPU selection vs the oracle's scores under the stated rule: exact where the k-th and
    (k+1)-th scores are more than 1e-3 apart; otherwise everything clearly above the cut is
    in, nothing clearly below it is."""
    F = len(scores_oracle)
    ref = O.topk_frames(scores_oracle, k)
    got = np.asarray(idx_gpu)
    n = min(k, F)
    assert (got[n:] == -1).all()
    got = got[:n]
    assert (np.diff(got) > 0).all()                     # ascending, hence distinct
    if n == F:
        np.testing.assert_array_equal(got, np.arange(F))
        return
    srt = np.sort(scores_oracle)[::-1]
    if srt[n - 1] - srt[n] > gap:
        np.testing.assert_array_equal(got, ref)
    else:
        cut = srt[n - 1]
        assert set(np.nonzero(scores_oracle > cut + gap)[0]) <= set(got)
        assert not (set(np.nonzero(scores_oracle < cut - gap)[0]) & set(got))


# ----------------------------------------------------------------------------------------
# C0: the whole tiny fp32 stream, every step of the path
# ----------------------------------------------------------------------------------------
def test_c0_whole_path_fp32():
    w = W.C0
    q, k, v = W.frames_q(w, 0, w.n_frames), W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    r = Rekv.for_workload(w)
    dq, dk, dv = dev(q, w), dev(k, w), dev(v, w)
    n_chunks = w.n_frames // w.chunk_frames
    out = r.encode_chunk(dq, dk, dv, 0, w.l_x, n_chunks, w.l_l)
    ref = O.encode_chunks(q, k, v, 0, w.l_x, n_chunks, w.l_l)
    assert np.abs(host(out) - ref).max() < TOL["f32"]
    # chunk by chunk gives the same as one call
    out2 = torch.cat([r.encode_chunk(dq[c * w.l_x:(c + 1) * w.l_x], dk, dv, c * w.l_x, w.l_x, 1, w.l_l)
                      for c in range(n_chunks)])
    assert torch.equal(out, out2)

    fk = r.frame_keys(dk, w.n_frames)
    fk_ref = O.frame_keys(k, w.n_frames, w.tokens_per_frame)
    assert np.abs(host(fk) - fk_ref).max() < 1e-5

    qq, qk, qv = W.question_qkv(w)
    idx, n_sel, scores = r.retrieve_topk(fk, w.n_frames, dev(qq, w)[None], w.top_k, want_scores=True)
    ref_idx, ref_s = O.retrieve(fk_ref, qq, w.n_kv_heads, w.top_k)
    assert np.abs(host(scores)[0] - ref_s).max() < 1e-5
    assert int(n_sel[0]) == w.top_k
    check_topk(idx[0].cpu().numpy(), ref_s, w.top_k)
    assert int(scores[0].argmax()) == 7 and 7 in idx[0].tolist()      # the planted frame

    gk, gv = r.gather_kv(dk, dv, idx)
    rk, rv = O.gather_kv(k, v, ref_idx, w.tokens_per_frame)
    assert gk.shape == (1, 64, 1, 64)
    assert host(gk)[0].tobytes() == rk.astype(np.float64).tobytes()
    assert host(gv)[0].tobytes() == rv.astype(np.float64).tobytes()

    o = r.qa_attention(dev(qq, w)[None], gk, gv, dev(qk, w)[None], dev(qv, w)[None])
    o_ref = O.qa_attention(qq, rk, rv, qk, qv)
    assert np.abs(host(o)[0] - o_ref).max() < TOL["f32"]


# ----------------------------------------------------------------------------------------
# encode, Eq. 1
# ----------------------------------------------------------------------------------------
ENCODE_CASES = [
    # name, workload, n_frames, chunk_frames, window_frames(None = tokens below), l_l tokens, chunks to check
    ("7B-ragged", W.C1, 20, 1, 16, None, [0, 1, 15, 16, 19]),
    ("7B-window-not-tile-multiple", W.C1, 6, 1, None, 250, [0, 2, 5]),
    ("7B-no-window", W.C1, 3, 1, None, 0, [0, 2]),
    ("7B-chunk-of-4-frames", W.C1, 12, 4, None, 1000, [0, 1, 2]),
    ("0.5B-D64", W.C1.scaled(n_q_heads=14, n_kv_heads=2, head_dim=64, name="C1-0.5B"), 8, 1, 4, None, [0, 3, 4, 7]),
    ("72B-G8", W.C4, 6, 1, 4, None, [0, 4, 5]),
    ("f32-D64-ragged", W.C0.scaled(tokens_per_frame=37, n_q_heads=6, n_kv_heads=2, name="C0r"), 9, 1, None, 100, [0, 3, 8]),
    ("f32-D128", W.C0.scaled(head_dim=128, tokens_per_frame=20, name="C0d"), 6, 2, None, 50, [0, 1, 2]),
]


@pytest.mark.parametrize("case", ENCODE_CASES, ids=[c[0] for c in ENCODE_CASES])
def test_encode_matches_oracle(case):
    _, w0, n_frames, chunk_frames, win_frames, l_l, chunks = case
    w = w0.scaled(n_frames=n_frames, chunk_frames=chunk_frames)
    l_l = win_frames * w.tokens_per_frame if l_l is None else l_l
    q, k, v = W.frames_q(w, 0, n_frames), W.frames_k(w, 0, n_frames), W.frames_v(w, 0, n_frames)
    r = Rekv.for_workload(w)
    n_chunks = n_frames // chunk_frames
    dq, dk, dv = dev(q, w), dev(k, w), dev(v, w)
    out = host(r.encode_chunk(dq, dk, dv, 0, w.l_x, n_chunks, l_l))
    assert np.isfinite(out).all()
    for c in chunks:
        sl = slice(c * w.l_x, (c + 1) * w.l_x)
        ref = O.encode_chunks(q[sl], k, v, c * w.l_x, w.l_x, 1, l_l)
        err = np.abs(out[sl] - ref).max()
        assert err < TOL[w.dtype], (c, err)
        # one chunk per call: few workgroups, so the key range is split over several of
        # them and merged - must agree with the oracle as well
        one = host(r.encode_chunk(dq[sl], dk, dv, c * w.l_x, w.l_x, 1, l_l))
        err = np.abs(one - ref).max()
        assert err < TOL[w.dtype], ("single", c, err)


def _random_encode_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        hkv = int(rng.choice([1, 2, 4]))
        g = int(rng.choice([1, 2, 3, 5, 7, 8]))
        cases.append(dict(dtype=str(rng.choice(["bf16", "bf16", "f32"])), hkv=hkv, hq=hkv * g,
                          d=int(rng.choice([64, 128])), nf=int(rng.integers(1, 71)),
                          chunk_frames=int(rng.integers(1, 4)), n_chunks=int(rng.integers(1, 5)),
                          first_chunk=int(rng.integers(0, 4)), l_l=int(rng.choice([0, 1, 31, 32, 33, 100, 257, 10 ** 6])),
                          seed=i))
    return cases


@pytest.mark.parametrize("c", _random_encode_cases(24, 2024), ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_encode_random_shapes(c):
    """Seeded sweep over head layouts, head sizes, frame sizes that are no multiple of anything,
    window lengths around the 32-key tile, calls that start in mid-stream and hold several chunks;
    every output row is compared."""
    w = W.C1.scaled(dtype=c["dtype"], n_q_heads=c["hq"], n_kv_heads=c["hkv"], head_dim=c["d"],
                    tokens_per_frame=c["nf"], chunk_frames=c["chunk_frames"],
                    n_frames=(c["first_chunk"] + c["n_chunks"]) * c["chunk_frames"], name=f"rnd{c['seed']}")
    q, k, v = W.frames_q(w, 0, w.n_frames), W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    r = Rekv.for_workload(w)
    t0 = c["first_chunk"] * w.l_x
    sl = slice(t0, t0 + c["n_chunks"] * w.l_x)
    out = host(r.encode_chunk(dev(q[sl], w), dev(k, w), dev(v, w), t0, w.l_x, c["n_chunks"], c["l_l"]))
    ref = O.encode_chunks(q[sl], k, v, t0, w.l_x, c["n_chunks"], c["l_l"])
    err = np.abs(out - ref).max()
    assert err < TOL[w.dtype], err


def test_encode_single_token_chunks_and_custom_scale():
    """l_x = 1 (a chunk is one token) and a caller-given softmax scale."""
    w = W.C1.scaled(n_frames=3)
    q, k, v = W.frames_q(w, 0, 3), W.frames_k(w, 0, 3), W.frames_v(w, 0, 3)
    r = Rekv.for_workload(w, softmax_scale=0.05)
    T = 3 * w.tokens_per_frame
    out = host(r.encode_chunk(dev(q, w)[400:], dev(k, w), dev(v, w), 400, 1, T - 400, 300))
    ref = O.encode_chunks(q[400:], k, v, 400, 1, T - 400, 300, scale=0.05)
    assert np.abs(out - ref).max() < TOL["bf16"]


def test_encode_rejects_bad_arguments():
    w = W.C1.scaled(n_frames=2)
    r = Rekv.for_workload(w)
    q, k = dev(W.frames_q(w, 0, 1), w), dev(W.frames_k(w, 0, 2), w)
    with pytest.raises(RekvError, match="INVALID_ARG"):
        r._check(r._lib.rekv_encode_chunk(r._h, q.data_ptr(), k.data_ptr(), k.data_ptr(), 0, 0, 1, 0,
                                          q.data_ptr(), None))
    with pytest.raises(RekvError, match="INVALID_ARG"):
        r._check(r._lib.rekv_encode_chunk(r._h, q.data_ptr(), None, k.data_ptr(), 0, 196, 1, 0,
                                          q.data_ptr(), None))
    with pytest.raises(RekvError, match="aligned"):
        r._check(r._lib.rekv_encode_chunk(r._h, q.data_ptr() + 2, k.data_ptr(), k.data_ptr(), 0, 195, 1, 0,
                                          q.data_ptr(), None))
    with pytest.raises(ValueError):
        r.encode_chunk(q, k, k, 196, 196, 2, 0)        # cache too short for two chunks


# ----------------------------------------------------------------------------------------
# frame vectors, scores, top-k
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("w", [W.C1.scaled(n_frames=37), W.C4.scaled(n_frames=21),
                               W.C1.scaled(n_q_heads=14, n_kv_heads=2, head_dim=64, n_frames=9, name="0.5B"),
                               W.C0.scaled(tokens_per_frame=5, n_frames=11, name="C0r")],
                         ids=["7B", "72B", "0.5B", "f32"])
def test_frame_keys_match_oracle(w):
    k = W.frames_k(w, 0, w.n_frames)
    r = Rekv.for_workload(w)
    fk = host(r.frame_keys(dev(k, w), w.n_frames))
    assert np.abs(fk - O.frame_keys(k, w.n_frames, w.tokens_per_frame)).max() < 1e-5
    # a prefix of the frames
    fk3 = host(r.frame_keys(dev(k, w), 3))
    np.testing.assert_array_equal(fk3, fk[:3])


@pytest.mark.parametrize("w,nq", [(W.C1.scaled(n_frames=300), 1), (W.C4.scaled(n_frames=130), 19),
                                  (W.C2.scaled(n_frames=1000), 3)], ids=["7B", "72B-19q", "hour-64"])
def test_retrieval_matches_oracle(w, nq):
    k = W.frames_k(w, 0, w.n_frames)
    fk_ref = O.frame_keys(k, w.n_frames, w.tokens_per_frame)
    r = Rekv.for_workload(w)
    fk = r.frame_keys(dev(k, w), w.n_frames)
    qs = [W.question_qkv(w, i)[0] for i in range(nq)]
    dq = dev(np.stack(qs), w)
    n_vis = w.n_frames - 7                              # the question's timestamp hides 7 frames
    idx, n_sel, scores = r.retrieve_topk(fk, n_vis, dq, w.top_k, want_scores=True)
    idx2, _, none = r.retrieve_topk(fk, n_vis, dq, w.top_k)            # scores kept internal
    assert none is None and torch.equal(idx, idx2)
    for i in range(nq):
        ref_idx, ref_s = O.retrieve(fk_ref, qs[i], w.n_kv_heads, w.top_k, n_visible=n_vis)
        assert np.abs(host(scores)[i] - ref_s).max() < 1e-5
        check_topk(idx[i].cpu().numpy(), ref_s, w.top_k)
        # the selection itself is exact given the scores it saw (ties to the lower index)
        np.testing.assert_array_equal(idx[i].cpu().numpy(), O.topk_frames(host(scores)[i], w.top_k))
        planted = [p for p in W.planted_frames(w, i) if p < n_vis]
        assert set(planted) <= set(idx[i].tolist())
        assert int(n_sel[i]) == w.top_k


# ----------------------------------------------------------------------------------------
# external retrieval scoring (Eq. 2 with tau on given embeddings)
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("dim,n_frames,nq,tau,k", [(768, 3600, 1, 0.07, 64), (1152, 1000, 5, 0.01, 16),
                                                   (64, 37, 9, 1.0, 50), (4, 3, 1, 2.5, 1)],
                         ids=["768-hour", "1152-5q", "tiny-k>F", "dim4"])
def test_external_retrieval_matches_oracle(dim, n_frames, nq, tau, k):
    """Embeddings of the sizes a CLIP-like encoder pair gives, drawn at random with a few frames
    pulled towards each question; scores and thresholds scale with 1 / tau."""
    rng = np.random.default_rng(dim + n_frames)
    emb = rng.standard_normal((n_frames, dim)).astype(np.float32)
    qe = rng.standard_normal((nq, dim)).astype(np.float32)
    for i in range(nq):
        for f in rng.choice(n_frames, size=min(3, n_frames), replace=False):
            emb[f] += 0.5 * qe[i]
    if n_frames > 5:
        emb[5] = 0.0                                                     # a zero-norm frame scores 0
    r = Rekv.for_workload(W.C1)
    idx, n_sel, scores = r.retrieve_external(torch.from_numpy(emb).to(DEV), torch.from_numpy(qe).to(DEV), k,
                                             tau=tau, want_scores=True)
    idx2, _, _ = r.retrieve_external(torch.from_numpy(emb).to(DEV), torch.from_numpy(qe).to(DEV), k, tau=tau)
    assert torch.equal(idx, idx2)
    for i in range(nq):
        ref_idx, ref_s = O.retrieve_external(emb, qe[i], k, tau)
        assert np.abs(host(scores)[i] - ref_s).max() < 1e-5 / tau
        check_topk(idx[i].cpu().numpy(), ref_s, k, gap=1e-3 / tau)
        np.testing.assert_array_equal(idx[i].cpu().numpy()[:min(k, n_frames)],
                                      O.topk_frames(host(scores)[i], k))
        assert int(n_sel[i]) == min(k, n_frames)
        if n_frames > 5:
            assert host(scores)[i][5] == 0.0
    with pytest.raises(RekvError):
        r.retrieve_external(torch.from_numpy(emb).to(DEV), torch.from_numpy(qe).to(DEV), k, tau=0.0)
    with pytest.raises(RekvError):
        r.retrieve_external(torch.zeros((4, 6), device=DEV), torch.zeros((1, 6), device=DEV), 1)   # dim % 4


def test_external_retrieval_random_shapes_sweep():
    """Sixteen random (dim, frames, questions, k, tau): vector lengths that are no multiple of the
    scoring kernels' column slabs, frame and question counts that leave ragged tiles, one question or
    many on the shared table."""
    rng = np.random.default_rng(2024)
    r = Rekv.for_workload(W.C1)
    for case in range(16):
        dim = 4 * int(rng.integers(1, 330))
        n_frames = int(rng.integers(1, 3000))
        nq = int(rng.choice([1, 2, 3, 4, 5, 31, 33, 70]))
        k = int(rng.integers(1, 70))
        tau = float(rng.choice([1.0, 0.07, 0.5]))
        emb = rng.standard_normal((n_frames, dim)).astype(np.float32)
        qe = rng.standard_normal((nq, dim)).astype(np.float32)
        print(f"case {case}: dim {dim}, {n_frames} frames, {nq} question(s), k {k}, tau {tau}", flush=True)
        idx, n_sel, scores = r.retrieve_external(torch.from_numpy(emb).to(DEV), torch.from_numpy(qe).to(DEV), k,
                                                 tau=tau, want_scores=True)
        sc = host(scores)
        for i in range(nq):
            _, ref_s = O.retrieve_external(emb, qe[i], k, tau)
            assert np.abs(sc[i] - ref_s).max() < 1e-5 / tau, (case, i)
            check_topk(idx[i].cpu().numpy(), ref_s, k, gap=1e-3 / tau)
            np.testing.assert_array_equal(idx[i].cpu().numpy()[:min(k, n_frames)], O.topk_frames(sc[i], k))
            assert int(n_sel[i]) == min(k, n_frames)


@pytest.mark.parametrize("n_frames,k", [(4097, 64), (10000, 1), (10000, 4096), (70000, 333)],
                         ids=["just-past-the-resident-limit", "k1", "largest-k", "70k-frames"])
def test_topk_on_tables_longer_than_the_resident_limit(n_frames, k):
    """More than 4,096 rows: the selection re-reads the scores from memory in every pass
    instead of keeping keys in LDS.  Includes the largest k the call accepts."""
    rng = np.random.default_rng(n_frames + k)
    emb = rng.standard_normal((n_frames, 32)).astype(np.float32)
    emb[::7] = emb[3]                                   # plenty of exact ties, also across the cut
    qe = rng.standard_normal((2, 32)).astype(np.float32)
    r = Rekv.for_workload(W.C1)
    idx, n_sel, scores = r.retrieve_external(torch.from_numpy(emb).to(DEV), torch.from_numpy(qe).to(DEV), k,
                                             want_scores=True)
    for i in range(2):
        ref_idx, ref_s = O.retrieve_external(emb, qe[i], k)
        s_gpu = host(scores)[i]
        assert np.abs(s_gpu - ref_s).max() < 1e-5
        np.testing.assert_array_equal(idx[i].cpu().numpy(), O.topk_frames(s_gpu, k))   # exact on its own scores
        check_topk(idx[i].cpu().numpy(), ref_s, k)
        assert int(n_sel[i]) == k
    with pytest.raises(RekvError):
        r.retrieve_external(torch.from_numpy(emb).to(DEV), torch.from_numpy(qe).to(DEV), 4097)


# ----------------------------------------------------------------------------------------
# block-level retrieval
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("b", [1, 2, 4, 8, 16])
def test_block_retrieval_hour_long_table(b):
    """The block-size ablation's setting (r = 64, b in 1..16) on a table as long as the
    hour-long stream's: 3,600 frame vectors of 512 dims, drawn directly (the frame-vector
    step has its own test), with a run of frames near each question so that something stands
    out.  3,600 is not a multiple of 16 or 32: b = 16 has a full last block, see the ragged
    case below for the short one."""
    w = W.C2
    F, dp, r_frames, nq = 3600, w.d_prime, 64, 3
    rng = np.random.default_rng(1000 + b)
    table = rng.standard_normal((F, dp)).astype(np.float32)
    qs = []
    for i in range(nq):
        q = rng.standard_normal((w.n_q_tokens, w.n_q_heads, w.head_dim))
        qv = O.question_vector(q, w.n_kv_heads)
        lo = 200 + 1000 * i
        table[lo:lo + 24] += (8.0 * qv).astype(np.float32)
        qs.append(W.round_to_bf16(q))
    r = Rekv.for_workload(w)
    t_dev = torch.from_numpy(table).to(DEV)
    bk = r.block_keys(t_dev, F, b)
    bk_ref = O.block_vectors(table, b)
    assert bk.shape[0] == bk_ref.shape[0] == -(-F // b)
    assert np.abs(host(bk) - bk_ref).max() < 1e-5
    kb = -(-r_frames // b)
    blk, n_blk, scores = r.retrieve_topk(bk, bk.shape[0], dev(np.stack(qs), w), kb, want_scores=True)
    fidx, n_sel = r.expand_blocks(blk, b, F)
    assert fidx.shape == (nq, kb * b)
    for i in range(nq):
        ref_frames, ref_blocks, ref_s = O.retrieve_blocks(table, qs[i], w.n_kv_heads, r_frames, b)
        assert np.abs(host(scores)[i] - ref_s).max() < 1e-5
        check_topk(blk[i].cpu().numpy(), ref_s, kb)
        got_blocks = blk[i].cpu().numpy()
        np.testing.assert_array_equal(fidx[i].cpu().numpy(), O.expand_blocks(got_blocks, b, F))
        assert int(n_sel[i]) == kb * b and int(n_blk[i]) == kb
        lo = 200 + 1000 * i                      # the planted run's fully covered blocks are in
        inside = [j for j in range(F // b) if j * b >= lo and (j + 1) * b <= lo + 24]
        assert set(inside) <= set(got_blocks.tolist())


def test_block_retrieval_ragged_stream_end_to_end():
    """Frames -> frame vectors -> block vectors -> block top-k -> frame list -> gather, on a
    stream whose last block is short and is the one the question points at."""
    b, r_frames = 8, 20
    w = W.C1.scaled(n_frames=59, tokens_per_frame=12, n_q_tokens=9, name="C1-blocks")
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    fk_ref = O.frame_keys(k, w.n_frames, w.tokens_per_frame)
    # the question: near the mean key of the last three frames (the short block 7 = frames 56..58)
    rng = np.random.default_rng(77)
    target = fk_ref[56:59].mean(axis=0).reshape(w.n_kv_heads, w.head_dim)
    q = np.repeat(target, w.group, axis=0)[None] + 0.3 * rng.standard_normal((w.n_q_tokens, w.n_q_heads, w.head_dim))
    q = W.round_to_bf16(q)
    r = Rekv.for_workload(w)
    dk, dv = dev(k, w), dev(v, w)
    fk = r.frame_keys(dk, w.n_frames)
    bk = r.block_keys(fk, w.n_frames, b)
    bk_ref = O.block_vectors(fk_ref, b)
    assert bk.shape[0] == 8 and np.abs(host(bk) - bk_ref).max() < 1e-5
    kb = -(-r_frames // b)                                                    # 3 blocks
    blk, _, scores = r.retrieve_topk(bk, 8, dev(q[None], w), kb, want_scores=True)
    ref_frames, ref_blocks, ref_s = O.retrieve_blocks(fk_ref, q, w.n_kv_heads, r_frames, b)
    assert np.abs(host(scores)[0] - ref_s).max() < 1e-5
    check_topk(blk[0].cpu().numpy(), ref_s, kb)
    assert 7 in blk[0].tolist() and 7 in ref_blocks.tolist()
    fidx, n_sel = r.expand_blocks(blk, b, w.n_frames)
    got = fidx[0].cpu().numpy()
    n = int(n_sel[0])
    assert n == 2 * b + 3 and (got[n:] == -1).all()
    np.testing.assert_array_equal(got[:n], O.expand_blocks(blk[0].cpu().numpy(), b, w.n_frames))
    gk, gv = r.gather_kv(dk, dv, fidx, n_src_frames=w.n_frames)
    rk, rv = O.gather_kv(k, v, got[:n], w.tokens_per_frame)
    nt = n * w.tokens_per_frame
    np.testing.assert_array_equal(host(gk)[0, :nt], rk)
    np.testing.assert_array_equal(host(gv)[0, :nt], rv)
    assert not host(gk)[0, nt:].any() and not host(gv)[0, nt:].any()       # -1 slots are zero-filled
    # more blocks asked for than the stream has: all frames, once, then -1
    blk_all, n_blk, _ = r.retrieve_topk(bk, 8, dev(q[None], w), 11)
    fidx, n_sel = r.expand_blocks(blk_all, b, w.n_frames)
    assert int(n_blk[0]) == 8 and int(n_sel[0]) == w.n_frames
    np.testing.assert_array_equal(fidx[0, :w.n_frames].cpu().numpy(), np.arange(w.n_frames))
    assert (fidx[0, w.n_frames:] == -1).all()
    with pytest.raises(RekvError):
        r.block_keys(fk, w.n_frames, 0)


def test_per_layer_tables_retrieve_independently():
    """Each 'question' row has its own frame-key table (one per layer)."""
    w = W.C3.scaled(n_frames=40, n_layers=3)
    r = Rekv.for_workload(w)
    fks, qs, refs = [], [], []
    for layer in range(3):
        k = W.frames_k(w, 0, w.n_frames, layer)
        fks.append(r.frame_keys(dev(k, w), w.n_frames))
        qq = W.question_qkv(w, 0, layer)[0]
        qs.append(qq)
        refs.append(O.retrieve(O.frame_keys(k, w.n_frames, w.tokens_per_frame), qq, w.n_kv_heads, w.top_k))
    table = torch.stack(fks)                                        # [layers, F, D']
    idx, _, scores = r.retrieve_topk(table, w.n_frames, dev(np.stack(qs), w), w.top_k,
                                     frame_keys_stride=w.n_frames * w.d_prime, want_scores=True)
    for layer in range(3):
        assert np.abs(host(scores)[layer] - refs[layer][1]).max() < 1e-5
        check_topk(idx[layer].cpu().numpy(), refs[layer][1], w.top_k)
    assert not torch.equal(idx[0], idx[1])


def test_topk_ties_and_degenerate_sizes():
    w = W.C0.scaled(n_frames=300, tokens_per_frame=2, name="ties")
    r = Rekv.for_workload(w)
    k = W.frames_k(w, 0, w.n_frames)
    k[40:] = np.tile(k[:40], (15, 1, 1))[: len(k) - 40]     # frames repeat with period 20: exact ties
    fk = r.frame_keys(dev(k, w), w.n_frames)
    qq = W.question_qkv(w)[0]
    # 300 frames go through the radix select; 200 and 64 through the one-pass count for small
    # tables, where a tie group straddling the cut (k = 15, 17, ...) must hand over to the radix select
    for n_vis in (300, 200, 64):
        for kk in (1, 2, 15, 16, 17, 64, 199, 200, 299, 300, 301, 500):
            idx, n_sel, scores = r.retrieve_topk(fk, n_vis, dev(qq, w)[None], kk, want_scores=True)
            s = host(scores)[0]
            assert len(np.unique(s)) <= 21
            ref = O.topk_frames(s, kk)
            got = idx[0].cpu().numpy()
            np.testing.assert_array_equal(got[: len(ref)], ref)
            assert (got[len(ref):] == -1).all() and int(n_sel[0]) == min(kk, n_vis)
    # zero keys and a zero question score 0 everywhere: the first k frames win
    z = torch.zeros_like(fk)
    idx, _, scores = r.retrieve_topk(z, 300, dev(qq, w)[None], 5, want_scores=True)
    assert idx[0].tolist() == [0, 1, 2, 3, 4] and float(scores.abs().max()) == 0.0
    # a single visible frame
    idx, n_sel, _ = r.retrieve_topk(fk, 1, dev(qq, w)[None], 4)
    assert idx[0].tolist() == [0, -1, -1, -1] and int(n_sel[0]) == 1
    with pytest.raises(RekvError, match="INVALID_ARG"):
        r.retrieve_topk(fk, 300, dev(qq, w)[None], 0)


# ----------------------------------------------------------------------------------------
# gather (device and pinned-host source), offload
# ----------------------------------------------------------------------------------------
def test_gather_device_and_host_bit_exact():
    w = W.C1.scaled(n_frames=24)
    r = Rekv.for_workload(w)
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    dk, dv = dev(k, w), dev(v, w)
    sel = np.array([[0, 3, 4, 5, 23], [1, 2, 9, -1, -1]], dtype=np.int32)
    idx = torch.from_numpy(sel).to(DEV)
    gk, gv = r.gather_kv(dk, dv, idx)
    hk = torch.empty(dk.shape, dtype=dk.dtype, pin_memory=True)
    hv = torch.empty(dv.shape, dtype=dv.dtype, pin_memory=True)
    r.offload_kv(dk, dv, hk, hv, 0, 10)                  # offload in two pieces
    r.offload_kv(dk, dv, hk, hv, 10, 14)
    r.offload_wait()
    assert torch.equal(hk, dk.cpu()) and torch.equal(hv, dv.cpu())
    for mode in (1, 2):                                  # copy-engine path, zero-copy kernel path
        gk_h, gv_h = r.gather_kv(hk, hv, idx, host_mode=mode)
        torch.cuda.synchronize()
        assert torch.equal(gk, gk_h) and torch.equal(gv, gv_h), mode
    nf = w.tokens_per_frame
    for qi in range(2):
        frames = [f for f in sel[qi] if f >= 0]
        rk, rv = O.gather_kv(k, v, frames, nf)
        n = len(frames) * nf
        assert host(gk)[qi, :n].tobytes() == rk.astype(np.float64).tobytes()
        assert host(gv)[qi, :n].tobytes() == rv.astype(np.float64).tobytes()
        assert float(gk[qi, n:].abs().max() if n < gk.shape[1] else 0) == 0     # skipped slots are zero
    bad = torch.tensor([[0, 99]], dtype=torch.int32, device=DEV)
    with pytest.raises(RekvError, match="INVALID_ARG"):
        r.gather_kv(hk, hv, bad, host_mode=1)
    zk, _ = r.gather_kv(hk, hv, bad, host_mode=2)        # the kernel paths skip what is out of range
    torch.cuda.synchronize()
    assert torch.equal(zk[0, :nf], dk[:nf]) and float(zk[0, nf:].abs().max()) == 0
    with pytest.raises(RekvError, match="pinned"):
        r._check(r._lib.rekv_gather_kv(r._h, dk.cpu().data_ptr(), dk.cpu().data_ptr(), 2, 24, idx.data_ptr(),
                                       2, 5, gk.data_ptr(), gv.data_ptr(), None))


@pytest.mark.parametrize("w,layout,mode,src_rotated", [
    (W.C1, "half", "consecutive", False), (W.C1, "interleaved", "consecutive", True),
    (W.C1, "half", "static", True), (W.C4, "half", "consecutive", True),
    (W.C0.scaled(tokens_per_frame=7, name="C0r"), "half", "consecutive", True),
    (W.C0.scaled(tokens_per_frame=7, name="C0r"), "interleaved", "static", False)],
    ids=["7B-plain-cache", "7B-interleaved-rotated-cache", "7B-static", "72B", "f32", "f32-interleaved-static"])
def test_gather_with_position_policy_matches_oracle(w, layout, mode, src_rotated):
    """Keys turned to consecutive (or one static) position while they are gathered; the cache
    holds plain keys or keys rotated at stream positions around 700,000 (an hour-long stream),
    so the angles are large.  Values must be copied bit for bit; keys agree to one unit in the
    last place of the storage type (the oracle is fp64, the result is rounded once)."""
    w = w.scaled(n_frames=20)
    r = Rekv.for_workload(w)
    nf = w.tokens_per_frame
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    src_off = 700_000
    if src_rotated:
        k = O.apply_rope(k, src_off + np.arange(k.shape[0]), layout=layout)
        k = W.round_to_bf16(k) if w.dtype == "bf16" else k.astype(np.float32).astype(np.float64)
    idx = np.array([[17, 3, 4, 9, -1], [0, 19, 18, -1, -1]], dtype=np.int32)
    gk, gv = r.gather_kv_rope(dev(k, w), dev(v, w), torch.from_numpy(idx).to(DEV), mode=mode, pos_offset=35,
                              src_rotated=src_rotated, src_pos_offset=src_off, layout=layout)
    gk, gv = host(gk), host(gv)
    for i in range(2):
        frames = [f for f in idx[i] if f >= 0]
        n = len(frames) * nf
        rk, rv = O.gather_kv_rope(k, v, frames, nf, mode=mode, pos_offset=35, src_rotated=src_rotated,
                                  src_pos_offset=src_off, layout=layout)
        np.testing.assert_array_equal(gv[i, :n], rv)
        ulp = 2.0 ** -8 if w.dtype == "bf16" else 2.0 ** -22
        tol = ulp * np.abs(rk) + (1e-5 if w.dtype == "bf16" else 5e-5)
        assert (np.abs(gk[i, :n] - rk) <= tol).all(), np.abs(gk[i, :n] - rk).max()
        assert not gk[i, n:].any() and not gv[i, n:].any()               # -1 slots are zero-filled
    with pytest.raises(RekvError):
        r.gather_kv_rope(dev(k, w), dev(v, w), torch.from_numpy(idx).to(DEV), base=1.0)


# ----------------------------------------------------------------------------------------
# QA attention, Eq. 3
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("w,nq,n_ret_frames", [
    (W.C1, 1, 16), (W.C1, 3, 5), (W.C1, 2, 0), (W.C4.scaled(n_q_tokens=17), 5, 3),
    (W.C2, 1, 64), (W.C0.scaled(tokens_per_frame=7, name="C0q"), 2, 3)],
    ids=["7B-k16", "7B-3q-k5", "no-retrieved", "72B-5q-ragged", "hour-k64", "f32"])
def test_qa_attention_matches_oracle(w, nq, n_ret_frames):
    w = w.scaled(n_frames=max(2 * n_ret_frames, 4))
    r = Rekv.for_workload(w)
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    nf = w.tokens_per_frame
    qs, ks, vs, rks, rvs = [], [], [], [], []
    for i in range(nq):
        qq, qk, qv = W.question_qkv(w, i)
        frames = list(range(i % 2, i % 2 + n_ret_frames))
        rk, rv = O.gather_kv(k, v, frames, nf)
        qs.append(qq); ks.append(qk); vs.append(qv); rks.append(rk); rvs.append(rv)
    shape_ret = (nq, n_ret_frames * nf, w.n_kv_heads, w.head_dim)
    out = r.qa_attention(dev(np.stack(qs), w), dev(np.stack(rks).reshape(shape_ret), w),
                         dev(np.stack(rvs).reshape(shape_ret), w), dev(np.stack(ks), w), dev(np.stack(vs), w))
    out = host(out)
    for i in range(nq):
        ref = O.qa_attention(qs[i], rks[i], rvs[i], ks[i], vs[i])
        err = np.abs(out[i] - ref).max()
        assert err < TOL[w.dtype], (i, err)


# ----------------------------------------------------------------------------------------
# answer decoding, Eq. 3 with X = the tokens being decoded
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("w,nq,n_ret_frames,n_gen,n_new,slack", [
    (W.C1, 1, 16, 20, 1, 12), (W.C1, 3, 5, 9, 4, 0), (W.C1, 2, 0, 0, 1, 3),
    (W.C4.scaled(n_q_tokens=17), 5, 3, 30, 1, 1), (W.C2, 1, 64, 128, 1, 0), (W.C1, 1, 16, 70, 40, 5),
    (W.C0.scaled(tokens_per_frame=7, name="C0d"), 2, 3, 6, 2, 2)],
    ids=["7B-k16", "7B-3q-4new", "no-retrieved", "72B-5q", "hour-k64-128gen", "7B-40new", "f32"])
def test_decode_attention_matches_oracle(w, nq, n_ret_frames, n_gen, n_new, slack):
    """Text KV = the question's tokens followed by n_gen generated ones; the last n_new are
    decoded.  Rows of the text buffers past the valid ones hold NaN: reading them would
    show in the output."""
    w = w.scaled(n_frames=max(2 * n_ret_frames, 4))
    r = Rekv.for_workload(w)
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    nf = w.tokens_per_frame
    n_text = w.n_q_tokens + n_gen
    stride = n_text + slack
    assert n_gen <= w.n_q_tokens * 4
    qs, kts, vts, rks, rvs = [], [], [], [], []
    for i in range(nq):
        parts = [W.question_qkv(w, i + 64 * j) for j in range(1 + (n_gen + w.n_q_tokens - 1) // w.n_q_tokens)]
        qt, kt, vt = (np.concatenate([p[c] for p in parts])[:n_text] for c in range(3))
        frames = list(range(i % 2, i % 2 + n_ret_frames))
        rk, rv = O.gather_kv(k, v, frames, nf)
        qs.append(qt[n_text - n_new:]); kts.append(kt); vts.append(vt); rks.append(rk); rvs.append(rv)
    pad = np.full((nq, slack, w.n_kv_heads, w.head_dim), np.nan)
    shape_ret = (nq, n_ret_frames * nf, w.n_kv_heads, w.head_dim)
    out = r.decode_attention(dev(np.stack(qs), w), dev(np.stack(rks).reshape(shape_ret), w),
                             dev(np.stack(rvs).reshape(shape_ret), w),
                             dev(np.concatenate([np.stack(kts), pad], axis=1), w),
                             dev(np.concatenate([np.stack(vts), pad], axis=1), w), n_text)
    out = host(out)
    assert np.isfinite(out).all()
    for i in range(nq):
        ref = O.decode_attention(qs[i], rks[i], rvs[i], kts[i], vts[i])
        err = np.abs(out[i] - ref).max()
        assert err < TOL[w.dtype], (i, err)


@pytest.mark.parametrize("w,nq,n_ret_frames,n_gen,n_new", [
    (W.C1, 1, 16, 0, None), (W.C1, 2, 16, 40, 1), (W.C4.scaled(n_q_tokens=17), 5, 7, 3, 2),
    (W.C1.scaled(tokens_per_frame=12, name="C1-12"), 3, 37, 0, None), (W.C2, 1, 64, 128, 1),
    (W.C0.scaled(tokens_per_frame=7, name="C0i"), 2, 5, 4, 2)],
    ids=["7B-prefill", "7B-decode", "72B-5q", "12-token-frames", "hour-k64-decode", "f32"])
def test_indexed_attention_matches_oracle_and_the_gathered_path(w, nq, n_ret_frames, n_gen, n_new):
    """Eq. 3 with the retrieved frames read in place through the index list: against the oracle
    (gather, then attention) and against this library's own gather + attention.  Frame lists
    are unsorted picks from a larger arena; the index rows are wider than the frames used and
    padded with -1."""
    w = w.scaled(n_frames=3 * n_ret_frames + 5)
    r = Rekv.for_workload(w)
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    nf = w.tokens_per_frame
    n_text = w.n_q_tokens + n_gen
    n_new = n_text if n_new is None else n_new
    rng = np.random.default_rng(5)
    idx = np.full((nq, n_ret_frames + 3), -1, dtype=np.int32)
    qs, kts, vts = [], [], []
    for i in range(nq):
        idx[i, :n_ret_frames] = rng.choice(w.n_frames, size=n_ret_frames, replace=False)
        parts = [W.question_qkv(w, i + 64 * j) for j in range(1 + (n_gen + w.n_q_tokens - 1) // w.n_q_tokens)]
        qt, kt, vt = (np.concatenate([p[c] for p in parts])[:n_text] for c in range(3))
        qs.append(qt[n_text - n_new:]); kts.append(kt); vts.append(vt)
    dk, dv = dev(k, w), dev(v, w)
    didx = torch.from_numpy(idx).to(DEV)
    dq, dkt, dvt = dev(np.stack(qs), w), dev(np.stack(kts), w), dev(np.stack(vts), w)
    out = r.attention_indexed(dq, dk, dv, didx, n_ret_frames, dkt, dvt, n_text)
    gk, gv = r.gather_kv(dk, dv, didx[:, :n_ret_frames].contiguous())
    via_gather = r.decode_attention(dq, gk, gv, dkt, dvt, n_text)
    assert (out.float() - via_gather.float()).abs().max().item() < 1e-6 + (4e-3 if w.dtype == "bf16" else 0)
    out = host(out)
    for i in range(nq):
        rk, rv = O.gather_kv(k, v, idx[i, :n_ret_frames], nf)
        ref = O.decode_attention(qs[i], rk, rv, kts[i], vts[i])
        err = np.abs(out[i] - ref).max()
        assert err < TOL[w.dtype], (i, err)
    # an entry outside the arena is clamped into it, never followed
    bad = didx.clone()
    bad[0, 0] = 2_000_000_000
    good = didx.clone()
    good[0, 0] = w.n_frames - 1
    a = r.attention_indexed(dq, dk, dv, bad, n_ret_frames, dkt, dvt, n_text)
    b = r.attention_indexed(dq, dk, dv, good, n_ret_frames, dkt, dvt, n_text)
    assert torch.equal(a, b)
    with pytest.raises(RekvError):
        r.attention_indexed(dq, dk, dv, didx, n_ret_frames + 4, dkt, dvt, n_text)     # wider than the index rows


def _random_qa_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        hkv = int(rng.choice([1, 2, 4, 8]))
        g = int(rng.choice([1, 2, 4, 7, 8]))
        n_text = int(rng.integers(1, 80))
        cases.append(dict(dtype=str(rng.choice(["bf16", "bf16", "f32"])), hkv=hkv, hq=hkv * g,
                          d=int(rng.choice([64, 128])), nf=int(rng.integers(1, 50)), nq=int(rng.integers(1, 4)),
                          n_ret=int(rng.integers(1, 20)), n_text=n_text, n_new=int(rng.integers(1, n_text + 1)),
                          slack=int(rng.integers(0, 5)), seed=i))
    return cases


@pytest.mark.parametrize("c", _random_qa_cases(24, 4242), ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_decode_and_indexed_attention_random_shapes(c):
    """Seeded sweep of Eq. 3 shapes: the same random case through the gathered path and through the
    in-place indexed path, both against the oracle, every output row."""
    w = W.C1.scaled(dtype=c["dtype"], n_q_heads=c["hq"], n_kv_heads=c["hkv"], head_dim=c["d"],
                    tokens_per_frame=c["nf"], n_frames=2 * c["n_ret"] + 3, name=f"rq{c['seed']}")
    rng = np.random.default_rng(c["seed"])
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    shape_q = (c["nq"], c["n_new"], w.n_q_heads, w.head_dim)
    shape_t = (c["nq"], c["n_text"], w.n_kv_heads, w.head_dim)
    rnd = lambda shape: (W.round_to_bf16(rng.standard_normal(shape)) if w.dtype == "bf16"
                         else rng.standard_normal(shape).astype(np.float32).astype(np.float64))
    q, kt, vt = rnd(shape_q), rnd(shape_t), rnd(shape_t)
    idx = np.stack([rng.choice(w.n_frames, size=c["n_ret"], replace=False) for _ in range(c["nq"])]).astype(np.int32)
    r = Rekv.for_workload(w)
    pad = np.full((c["nq"], c["slack"], w.n_kv_heads, w.head_dim), np.nan)
    dkt, dvt = dev(np.concatenate([kt, pad], axis=1), w), dev(np.concatenate([vt, pad], axis=1), w)
    dk, dv, didx = dev(k, w), dev(v, w), torch.from_numpy(idx).to(DEV)
    gk, gv = r.gather_kv(dk, dv, didx)
    a = host(r.decode_attention(dev(q, w), gk, gv, dkt, dvt, c["n_text"]))
    b = host(r.attention_indexed(dev(q, w), dk, dv, didx, c["n_ret"], dkt, dvt, c["n_text"]))
    for i in range(c["nq"]):
        rk, rv = O.gather_kv(k, v, idx[i], w.tokens_per_frame)
        ref = O.decode_attention(q[i], rk, rv, kt[i], vt[i])
        assert np.abs(a[i] - ref).max() < TOL[w.dtype]
        assert np.abs(b[i] - ref).max() < TOL[w.dtype]


def test_decode_attention_rejects_bad_arguments():
    w = W.C1
    r = Rekv.for_workload(w)
    q = torch.zeros((1, 2, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=DEV)
    kr = torch.zeros((1, 8, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16, device=DEV)
    kt = torch.zeros((1, 4, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(RekvError):
        r.decode_attention(q, kr, kr, kt, kt, 1)       # fewer text rows than new tokens
    with pytest.raises(RekvError):
        r.decode_attention(q, kr, kr, kt, kt, 5)       # more valid rows than the buffer holds


def test_probes_copy_is_exact_and_mfma_reports_its_work():
    r = Rekv.for_workload(W.C1)
    src = torch.randint(0, 255, (3 * 1024 * 1024 + 48,), dtype=torch.uint8, device=DEV)
    dst = torch.zeros_like(src)
    assert r.probe_copy(dst, src) == src.numel()
    assert torch.equal(dst, src)
    sink = torch.empty(8 * 256, dtype=torch.float32, device=DEV)
    flop = r.probe_mfma(sink, 8, 16)
    assert flop == 2.0 * 32 * 32 * 16 * 4 * 4 * 8 * 16
    assert torch.isfinite(sink).all()
    with pytest.raises(RekvError):
        r.probe_copy(dst[:40], src[:40])                # not a multiple of 16 bytes


# ----------------------------------------------------------------------------------------
# the benchmark's launch configuration at full size, on sampled chunks
# ----------------------------------------------------------------------------------------
def test_c1_full_size_sampled_chunks_and_retrieval():
    w = W.C1
    n_chunks = w.n_frames // w.chunk_frames
    q, k, v = W.frames_q(w, 0, w.n_frames), W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    r = Rekv.for_workload(w)
    dq, dk, dv = dev(q, w), dev(k, w), dev(v, w)
    out = r.encode_chunk(dq, dk, dv, 0, w.l_x, n_chunks, w.l_l)      # one call, as bench.py times it
    torch.cuda.synchronize()
    for c in W.parity_chunks(n_chunks, w.window_frames):
        sl = slice(c * w.l_x, (c + 1) * w.l_x)
        ref = O.encode_chunks(q[sl], k, v, c * w.l_x, w.l_x, 1, w.l_l)
        err = np.abs(host(out[sl]) - ref).max()
        assert err < TOL["bf16"], (c, err)
    fk = r.frame_keys(dk, w.n_frames)
    fk_ref = O.frame_keys(k, w.n_frames, w.tokens_per_frame)
    assert np.abs(host(fk) - fk_ref).max() < 1e-5
    qq, qk, qv = W.question_qkv(w)
    idx, _, scores = r.retrieve_topk(fk, w.n_frames, dev(qq, w)[None], w.top_k, want_scores=True)
    ref_idx, ref_s = O.retrieve(fk_ref, qq, w.n_kv_heads, w.top_k)
    check_topk(idx[0].cpu().numpy(), ref_s, w.top_k)
    assert set(W.planted_frames(w)) <= set(idx[0].tolist())
    gk, gv = r.gather_kv(dk, dv, idx)
    o = r.qa_attention(dev(qq, w)[None], gk, gv, dev(qk, w)[None], dev(qv, w)[None])
    rk, rv = O.gather_kv(k, v, idx[0].tolist(), w.tokens_per_frame)
    assert host(gk)[0].tobytes() == rk.astype(np.float64).tobytes()
    o_ref = O.qa_attention(qq, rk, rv, qk, qv)
    assert np.abs(host(o)[0] - o_ref).max() < TOL["bf16"]
