"""The large benchmark configurations at their real shapes: hour-long stream with KV in
pinned host memory, per-layer retrieval over 28-layer shapes, many concurrent questions at
72B-class shapes.  The oracle cannot run these whole, so parity is checked on sampled
chunks / layers / questions (each output is a pure function of the given Q/K/V) and on
properties that hold at any size.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

from oracle import rekv_oracle as O
from paper_2503_00540_amd import workloads as W
from paper_2503_00540_amd.rekv import Rekv

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-2


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16).to(DEV)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def blockwise(fn, w, n_frames, layer=0, step=256):
    return torch.cat([dev(fn(w, f, min(f + step, n_frames), layer)) for f in range(0, n_frames, step)])


def check_topk(idx_gpu, scores_oracle, k):
    ref = O.topk_frames(scores_oracle, k)
    got = np.asarray(idx_gpu)
    assert (np.diff(got) > 0).all()
    srt = np.sort(scores_oracle)[::-1]
    if srt[k - 1] - srt[k] > 1e-3:
        np.testing.assert_array_equal(got, ref)
    else:
        cut = srt[k - 1]
        assert set(np.nonzero(scores_oracle > cut + 1e-3)[0]) <= set(got)
        assert not (set(np.nonzero(scores_oracle < cut - 1e-3)[0]) & set(got))


def test_c2_hour_long_stream_with_host_kv():
    """3,600 frames; KV is offloaded to pinned host memory after encoding; only the frame
    vectors stay in HBM; retrieval scores all frames, gathers 64 frames from the host."""
    w = W.C2
    r = Rekv.for_workload(w)
    F, nf = w.n_frames, w.tokens_per_frame
    dk = blockwise(W.frames_k, w, F)
    dv = blockwise(W.frames_v, w, F)
    # streaming encode, one launch per chunk, on sampled chunks
    for c in (0, 17, 1800, 3599):
        q = W.frames_q(w, c, c + 1)
        out = r.encode_chunk(dev(q), dk, dv, c * nf, nf, 1, w.l_l)
        f0 = max(0, c - w.window_frames)
        k_np, v_np = W.frames_k(w, f0, c + 1), W.frames_v(w, f0, c + 1)
        ref = O.encode_chunks(q, k_np, v_np, (c - f0) * nf, nf, 1, w.l_l)
        assert np.abs(host(out) - ref).max() < TOL, c
    fk = r.frame_keys(dk, F)
    hk = torch.empty(dk.shape, dtype=dk.dtype, pin_memory=True)
    hv = torch.empty(dv.shape, dtype=dv.dtype, pin_memory=True)
    for f in range(0, F, 400):                       # offload as the stream advances
        r.offload_kv(dk, dv, hk, hv, f, min(400, F - f))
    r.offload_wait()
    k_np, v_np = hk.float().numpy(), hv.float().numpy()
    del dk, dv
    torch.cuda.empty_cache()
    fk_ref = O.frame_keys(k_np, F, nf)
    assert np.abs(host(fk) - fk_ref).max() < 1e-5
    qq, qk, qv = W.question_qkv(w)
    idx, n_sel, scores = r.retrieve_topk(fk, F, dev(qq)[None], w.top_k, want_scores=True)
    ref_idx, ref_s = O.retrieve(fk_ref, qq, w.n_kv_heads, w.top_k)
    assert np.abs(host(scores)[0] - ref_s).max() < 1e-5
    check_topk(idx[0].cpu().numpy(), ref_s, w.top_k)
    assert set(W.planted_frames(w)) <= set(idx[0].tolist()) and int(n_sel[0]) == 64
    gk, gv = r.gather_kv(hk, hv, idx)                # host -> HBM on the side stream
    sel = idx[0].tolist()
    rk, rv = O.gather_kv(k_np, v_np, sel, nf)
    assert host(gk)[0].tobytes() == rk.astype(np.float64).tobytes()
    assert host(gv)[0].tobytes() == rv.astype(np.float64).tobytes()
    o = r.qa_attention(dev(qq)[None], gk, gv, dev(qk)[None], dev(qv)[None])
    assert np.abs(host(o)[0] - O.qa_attention(qq, rk, rv, qk, qv)).max() < TOL


def test_c3_layers_retrieve_independently_at_full_frame_count():
    """28-layer shapes, chunk of 4 frames, window of 32 frames; three sampled layers, each
    with its own KV, frame-vector table and question; one retrieval call for all of them."""
    w = W.C3
    r = Rekv.for_workload(w)
    F, nf, layers = w.n_frames, w.tokens_per_frame, (0, 13, 27)
    n_chunks = F // w.chunk_frames
    tables, qs, refs, kvs = [], [], [], []
    for layer in layers:
        dk = blockwise(W.frames_k, w, F, layer)
        dv = blockwise(W.frames_v, w, F, layer)
        tables.append(r.frame_keys(dk, F))
        for c in (0, 9, n_chunks - 1):
            f_lo, f_hi = c * w.chunk_frames, (c + 1) * w.chunk_frames
            q = W.frames_q(w, f_lo, f_hi, layer)
            out = r.encode_chunk(dev(q), dk, dv, f_lo * nf, w.l_x, 1, w.l_l)
            f0 = max(0, f_lo - w.window_frames)
            ref = O.encode_chunks(q, W.frames_k(w, f0, f_hi, layer), W.frames_v(w, f0, f_hi, layer),
                                  (f_lo - f0) * nf, w.l_x, 1, w.l_l)
            assert np.abs(host(out) - ref).max() < TOL, (layer, c)
        k_np = host(dk).astype(np.float32)
        qq = W.question_qkv(w, 0, layer)
        qs.append(qq)
        refs.append(O.retrieve(O.frame_keys(k_np, F, nf), qq[0], w.n_kv_heads, w.top_k))
        kvs.append((dk, dv))
    table = torch.stack(tables)
    idx, _, scores = r.retrieve_topk(table, F, dev(np.stack([q[0] for q in qs])), w.top_k,
                                     frame_keys_stride=F * w.d_prime, want_scores=True)
    for i, layer in enumerate(layers):
        assert np.abs(host(scores)[i] - refs[i][1]).max() < 1e-5
        check_topk(idx[i].cpu().numpy(), refs[i][1], w.top_k)
        assert set(W.planted_frames(w, 0, layer)) <= set(idx[i].tolist())
        dk, dv = kvs[i]
        gk, gv = r.gather_kv(dk, dv, idx[i:i + 1])
        sel = idx[i].tolist()
        rk = torch.cat([dk[f * nf:(f + 1) * nf] for f in sel])
        assert torch.equal(gk[0], rk)
        qq, qk, qv = qs[i]
        o = r.qa_attention(dev(qq)[None], gk, gv, dev(qk)[None], dev(qv)[None])
        ref = O.qa_attention(qq, host(gk)[0], host(gv)[0], qk, qv)
        assert np.abs(host(o)[0] - ref).max() < TOL
    assert not torch.equal(idx[0], idx[1])           # layers retrieve different frames


def test_c4_many_concurrent_questions():
    """72B-class shapes, 2,048 frames, 64 questions batched through scoring, top-k, gather
    and QA attention; oracle on sampled questions and chunks."""
    w = W.C4
    r = Rekv.for_workload(w)
    F, nf, nq = w.n_frames, w.tokens_per_frame, w.n_questions
    dk = blockwise(W.frames_k, w, F)
    dv = blockwise(W.frames_v, w, F)
    for c in (0, 16, 2047):
        q = W.frames_q(w, c, c + 1)
        out = r.encode_chunk(dev(q), dk, dv, c * nf, nf, 1, w.l_l)
        f0 = max(0, c - w.window_frames)
        ref = O.encode_chunks(q, W.frames_k(w, f0, c + 1), W.frames_v(w, f0, c + 1), (c - f0) * nf, nf, 1, w.l_l)
        assert np.abs(host(out) - ref).max() < TOL, c
    # eight chunks in one launch equal the single launches
    q8 = dev(W.frames_q(w, 100, 108))
    many = r.encode_chunk(q8, dk, dv, 100 * nf, nf, 8, w.l_l)
    one = r.encode_chunk(q8[3 * nf:4 * nf], dk, dv, 103 * nf, nf, 1, w.l_l)
    assert (many[3 * nf:4 * nf].float() - one.float()).abs().max() < TOL
    fk = r.frame_keys(dk, F)
    k_np = host(dk).astype(np.float32)
    fk_ref = O.frame_keys(k_np, F, nf)
    assert np.abs(host(fk) - fk_ref).max() < 1e-5
    qs = [W.question_qkv(w, i) for i in range(nq)]
    dq, dqk, dqv = (dev(np.stack([x[j] for x in qs])) for j in range(3))
    idx, n_sel, scores = r.retrieve_topk(fk, F, dq, w.top_k, want_scores=True)
    assert (n_sel == w.top_k).all()
    for i in range(nq):
        ref_idx, ref_s = O.retrieve(fk_ref, qs[i][0], w.n_kv_heads, w.top_k)
        assert np.abs(host(scores)[i] - ref_s).max() < 1e-5
        check_topk(idx[i].cpu().numpy(), ref_s, w.top_k)
        assert set(W.planted_frames(w, i)) <= set(idx[i].tolist())
    gk, gv = r.gather_kv(dk, dv, idx)
    o = r.qa_attention(dq, gk, gv, dqk, dqv)
    v_np = host(dv).astype(np.float32)
    for i in (0, 31, 63):
        sel = idx[i].tolist()
        rk, rv = O.gather_kv(k_np, v_np, sel, nf)
        assert host(gk)[i].tobytes() == rk.astype(np.float64).tobytes()
        assert host(gv)[i].tobytes() == rv.astype(np.float64).tobytes()
        ref = O.qa_attention(qs[i][0], rk, rv, qs[i][1], qs[i][2])
        assert np.abs(host(o)[i] - ref).max() < TOL, i


def test_retrieval_and_qa_replay_from_a_hip_graph():
    """The question-time part of the path (retrieval, gather, QA attention; and the variant that
    reads the retrieved frames in place) captured into a HIP graph: every replay, with eager work
    and synchronisations of the program in between, must give the eager result bit for bit.  The
    calls launch kernels only (no memset or copy nodes) once the context's workspace exists."""
    w = W.C1.scaled(n_frames=64)
    r = Rekv.for_workload(w)
    F = w.n_frames
    g = torch.Generator(device=DEV).manual_seed(11)
    mk = lambda *s: torch.randn(*s, device=DEV, generator=g).to(torch.bfloat16)
    k, v = mk(F * w.tokens_per_frame, w.n_kv_heads, w.head_dim), mk(F * w.tokens_per_frame, w.n_kv_heads, w.head_dim)
    qq = mk(2, w.n_q_tokens, w.n_q_heads, w.head_dim)
    qk, qv = mk(2, w.n_q_tokens, w.n_kv_heads, w.head_dim), mk(2, w.n_q_tokens, w.n_kv_heads, w.head_dim)
    fk = r.frame_keys(k, F)

    def gathered():
        idx, _, _ = r.retrieve_topk(fk, F, qq, w.top_k)
        gk, gv = r.gather_kv(k, v, idx, n_src_frames=F)
        return r.qa_attention(qq, gk, gv, qk, qv), idx

    def in_place():
        idx, _, _ = r.retrieve_topk(fk, F, qq, w.top_k)
        return r.attention_indexed(qq, k, v, idx, w.top_k, qk, qv, w.n_q_tokens, n_src_frames=F), idx

    for fn in (gathered, in_place):
        ref, ref_idx = fn()                              # eager; also grows the workspace before capture
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            out, idx = fn()
        for _ in range(4):
            out.zero_()
            idx.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, ref) and torch.equal(idx, ref_idx)
            scratch = r.frame_keys(k, F)                 # eager library work between replays
            assert torch.equal(scratch, fk)


def test_encode_with_the_papers_window_of_15k_tokens():
    """The experiments' setting: local window of 15K tokens (neither a multiple of the 196-token
    frame nor of the kernel's 32-key tile), one frame per chunk, 7B head layout.  Checked on
    chunks before and after the window fills, one call for the stream and one call per chunk."""
    w = W.C1.scaled(n_frames=100, name="C1-15k")
    l_l = 15000
    q, k, v = W.frames_q(w, 0, w.n_frames), W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    r = Rekv.for_workload(w)
    dq, dk, dv = dev(q), dev(k), dev(v)
    out = host(r.encode_chunk(dq, dk, dv, 0, w.l_x, w.n_frames, l_l))
    for c in (76, 77, 99):                       # 76 * 196 = 14,896 < 15,000 <= 77 * 196
        sl = slice(c * w.l_x, (c + 1) * w.l_x)
        ref = O.encode_chunks(q[sl], k, v, c * w.l_x, w.l_x, 1, l_l)
        assert np.abs(out[sl] - ref).max() < TOL, c
        one = host(r.encode_chunk(dq[sl], dk, dv, c * w.l_x, w.l_x, 1, l_l))
        assert np.abs(one - ref).max() < TOL, ("single", c)
