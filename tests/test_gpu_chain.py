"""Chains of calls and stress cases of the HIP path against the CPU oracle: selections shorter
than k carried through gather / in-place attention, score ranges that force the running
softmax maximum to be renewed in every tile, multi-chunk launches at benchmark shapes, and the
ordering of the side stream behind long work on the caller's stream.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

from oracle import rekv_oracle as O
from paper_2503_00540_amd import workloads as W
from paper_2503_00540_amd.rekv import Rekv

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {"bf16": 2e-2, "f32": 1e-4}


def dev(x, w):
    t = torch.from_numpy(np.ascontiguousarray(x))
    return t.to(torch.bfloat16 if w.dtype == "bf16" else torch.float32).to(DEV)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


# ----------------------------------------------------------------------------------------
# Eq. 3 when fewer than k frames were selected: the padding must stay out of the softmax
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("w0", [W.C1, W.C0.scaled(n_q_heads=4, n_kv_heads=2, name="C0-2kv"),
                                W.C1.scaled(n_q_heads=14, n_kv_heads=2, head_dim=64, name="C1-0.5B")], ids=["bf16", "f32", "bf16-D64"])
def test_short_selections_through_gather_and_in_place_attention(w0):
    """Block retrieval on a stream whose last block is short: question 0 points at that block and
    gets fewer frames than question 1, in one batch.  retrieve -> expand -> gather -> QA attention
    (and decode, and the in-place variant) with n_sel must equal the oracle, which attends to the
    frames that exist only."""
    b, r_frames = 8, 20
    w = w0.scaled(n_frames=59, tokens_per_frame=12, n_q_tokens=9, name=w0.name + "-short")
    nf = w.tokens_per_frame
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    fk_ref = O.frame_keys(k, w.n_frames, nf)
    rng = np.random.default_rng(3)
    targets = [fk_ref[56:59].mean(axis=0), fk_ref[16:24].mean(axis=0)]      # short block 7; full block 2
    qs = []
    for t in targets:
        base = np.repeat(t.reshape(w.n_kv_heads, w.head_dim), w.group, axis=0)[None]
        q = base + 0.3 * rng.standard_normal((w.n_q_tokens, w.n_q_heads, w.head_dim))
        qs.append(W.round_to_bf16(q) if w.dtype == "bf16" else q.astype(np.float32).astype(np.float64))
    qk = rng.standard_normal((2, w.n_q_tokens, w.n_kv_heads, w.head_dim))
    qv = rng.standard_normal((2, w.n_q_tokens, w.n_kv_heads, w.head_dim))
    if w.dtype == "bf16":
        qk, qv = W.round_to_bf16(qk), W.round_to_bf16(qv)
    else:
        qk, qv = qk.astype(np.float32).astype(np.float64), qv.astype(np.float32).astype(np.float64)
    r = Rekv.for_workload(w)
    dk, dv = dev(k, w), dev(v, w)
    dq, dqk, dqv = dev(np.stack(qs), w), dev(qk, w), dev(qv, w)
    fk = r.frame_keys(dk, w.n_frames)
    bk = r.block_keys(fk, w.n_frames, b)
    kb = -(-r_frames // b)
    blk, _, _ = r.retrieve_topk(bk, bk.shape[0], dq, kb)
    fidx, n_sel = r.expand_blocks(blk, b, w.n_frames)
    n = n_sel.tolist()
    assert n[0] == 2 * b + 3, n                                  # the short block is among question 0's
    if w.dtype == "bf16":
        assert n[1] == 3 * b, n                                  # different counts inside one batch
    refs = []
    for i in range(2):
        frames, _, _ = O.retrieve_blocks(fk_ref, qs[i], w.n_kv_heads, r_frames, b)
        assert n[i] == len(frames)
        np.testing.assert_array_equal(fidx[i, :n[i]].cpu().numpy(), frames)
        assert (fidx[i, n[i]:] == -1).all()
        rk, rv = O.gather_kv(k, v, frames, nf)
        refs.append(O.qa_attention(qs[i], rk, rv, qk[i], qv[i]))
    gk, gv = r.gather_kv(dk, dv, fidx, n_src_frames=w.n_frames)
    out = host(r.qa_attention(dq, gk, gv, dqk, dqv, n_sel=n_sel))
    out_dec = host(r.decode_attention(dq, gk, gv, dqk, dqv, w.n_q_tokens, n_sel=n_sel))
    out_idx = host(r.attention_indexed(dq, dk, dv, fidx, fidx.shape[1], dqk, dqv, w.n_q_tokens,
                                       n_src_frames=w.n_frames, n_sel=n_sel))
    for i in range(2):
        for name, o in (("qa", out), ("decode", out_dec), ("indexed", out_idx)):
            err = np.abs(o[i] - refs[i]).max()
            assert err < TOL[w.dtype], (name, i, err)
    # without n_sel the zero-filled padding of question 0 takes part in the softmax: a different result
    diluted = host(r.qa_attention(dq, gk, gv, dqk, dqv))
    assert np.abs(diluted[0] - refs[0]).max() > np.abs(out[0] - refs[0]).max()
    if n[1] == kb * b:
        assert np.abs(diluted[1] - refs[1]).max() < TOL[w.dtype]     # question 1 has no padding


def test_young_stream_selection_of_everything():
    """k larger than the frames seen so far: all frames are selected, n_sel = F for every question,
    and the attention over the gathered (padded) buffer with n_sel equals the oracle's."""
    w = W.C4.scaled(n_frames=5, n_q_tokens=7, name="C4-young")
    nf, k_top = w.tokens_per_frame, 8
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    r = Rekv.for_workload(w)
    dk, dv = dev(k, w), dev(v, w)
    qs = [W.question_qkv(w, i, n_visible=w.n_frames) for i in range(3)]
    dq, dqk, dqv = (dev(np.stack([x[j] for x in qs]), w) for j in range(3))
    fk = r.frame_keys(dk, w.n_frames)
    idx, n_sel, _ = r.retrieve_topk(fk, w.n_frames, dq, k_top)
    assert n_sel.tolist() == [5, 5, 5] and (idx[:, 5:] == -1).all()
    gk, gv = r.gather_kv(dk, dv, idx, n_src_frames=w.n_frames)
    out = host(r.qa_attention(dq, gk, gv, dqk, dqv, n_sel=n_sel))
    out_idx = host(r.attention_indexed(dq, dk, dv, idx, k_top, dqk, dqv, w.n_q_tokens, n_src_frames=w.n_frames,
                                       n_sel=n_sel))
    for i in range(3):
        ref = O.qa_attention(qs[i][0], k, v, qs[i][1], qs[i][2])        # all five frames, in order
        assert np.abs(out[i] - ref).max() < TOL["bf16"], i
        assert np.abs(out_idx[i] - ref).max() < TOL["bf16"], i
    # n_sel = 0: only the question's own tokens
    zero = torch.zeros(3, dtype=torch.int32, device=DEV)
    out0 = host(r.qa_attention(dq, gk, gv, dqk, dqv, n_sel=zero))
    for i in range(3):
        ref = O.qa_attention(qs[i][0], k[:0], v[:0], qs[i][1], qs[i][2])
        assert np.abs(out0[i] - ref).max() < TOL["bf16"], i


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_random_selection_lengths_sweep(dtype):
    """Twelve random shapes per storage type: every question of a batch keeps a random number of its k
    list entries (none at all included), the rest is -1 padding.  Gathered QA attention, the decode
    step and the in-place variant against the oracle on the frames that are kept."""
    rng = np.random.default_rng(77 if dtype == "bf16" else 78)
    base = W.C1 if dtype == "bf16" else W.C0.scaled(n_q_heads=4, n_kv_heads=2, name="C0-2kv")
    for case in range(12):
        d = int(rng.choice([64, 128])) if dtype == "bf16" else int(rng.choice([32, 64, 128]))
        hkv = int(rng.choice([1, 2, 4]))
        group = int(rng.choice([1, 4, 7]))
        w = base.scaled(n_frames=int(rng.integers(6, 30)), tokens_per_frame=int(rng.integers(3, 45)),
                        n_q_tokens=int(rng.integers(1, 40)), n_q_heads=hkv * group, n_kv_heads=hkv, head_dim=d,
                        name=f"sweep-{dtype}-{case}")
        nf, nq, k = w.tokens_per_frame, int(rng.integers(1, 4)), int(rng.integers(1, 6))
        kf, vf = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
        idx = np.full((nq, k), -1, dtype=np.int32)
        keep = rng.integers(0, k + 1, size=nq)
        for i in range(nq):
            idx[i, :keep[i]] = np.sort(rng.choice(w.n_frames, size=keep[i], replace=False))
        shape_q = (nq, w.n_q_tokens, w.n_q_heads, d)
        shape_kv = (nq, w.n_q_tokens, hkv, d)
        q, qk, qv = rng.standard_normal(shape_q), rng.standard_normal(shape_kv), rng.standard_normal(shape_kv)
        if dtype == "bf16":
            q, qk, qv = W.round_to_bf16(q), W.round_to_bf16(qk), W.round_to_bf16(qv)
        else:
            q, qk, qv = (x.astype(np.float32).astype(np.float64) for x in (q, qk, qv))
        r = Rekv.for_workload(w)
        dk, dv, didx = dev(kf, w), dev(vf, w), torch.from_numpy(idx).to(DEV)
        n_sel = torch.from_numpy(keep.astype(np.int32)).to(DEV)
        dq, dqk, dqv = dev(q, w), dev(qk, w), dev(qv, w)
        print(f"case {w.name}: frames {w.n_frames} x {nf}, Hq/Hkv/D {w.n_q_heads}/{hkv}/{d}, {nq} question(s) of "
              f"{w.n_q_tokens}, k {k}, kept {keep.tolist()}", flush=True)
        gk, gv = r.gather_kv(dk, dv, didx, n_src_frames=w.n_frames)
        outs = {"qa": host(r.qa_attention(dq, gk, gv, dqk, dqv, n_sel=n_sel)),
                "decode": host(r.decode_attention(dq, gk, gv, dqk, dqv, w.n_q_tokens, n_sel=n_sel)),
                "indexed": host(r.attention_indexed(dq, dk, dv, didx, k, dqk, dqv, w.n_q_tokens,
                                                    n_src_frames=w.n_frames, n_sel=n_sel))}
        for i in range(nq):
            rk, rv = O.gather_kv(kf, vf, [int(f) for f in idx[i, :keep[i]]], nf)
            ref = O.qa_attention(q[i], rk, rv, qk[i], qv[i])
            for name, o in outs.items():
                err = np.abs(o[i] - ref).max()
                assert err < TOL[dtype], (w.name, name, i, int(keep[i]), err)


# ----------------------------------------------------------------------------------------
# the running maximum rises in every tile: the rescaling of partial sums is exercised
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("q_scale", [8.0, 32.0])
def test_encode_when_the_softmax_maximum_keeps_rising(q_scale):
    """Keys carry a component along one direction that grows with the key's position and queries
    point along it, scaled up: every 32-key tile's best score lies far above (more than 2^8 times)
    everything before it, so the accumulated output is rescaled in every tile.  One launch for all
    chunks, and one launch per chunk (key range split over workgroups, then merged)."""
    w = W.C1.scaled(n_frames=6, name="C1-rising")
    T = w.n_frames * w.tokens_per_frame
    q, k, v = W.frames_q(w, 0, w.n_frames), W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    rng = np.random.default_rng(9)
    u = rng.standard_normal((w.n_kv_heads, w.head_dim))
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    ramp = 0.3 * np.arange(T)[:, None, None]
    k = W.round_to_bf16(k + ramp * u[None])
    q = W.round_to_bf16(q_scale * (q + np.repeat(u, w.group, axis=0)[None]))
    l_l = 4 * w.tokens_per_frame
    r = Rekv.for_workload(w)
    dq, dk, dv = dev(q, w), dev(k, w), dev(v, w)
    out = host(r.encode_chunk(dq, dk, dv, 0, w.l_x, w.n_frames, l_l))
    assert np.isfinite(out).all()
    for c in range(w.n_frames):
        sl = slice(c * w.l_x, (c + 1) * w.l_x)
        ref = O.encode_chunks(q[sl], k, v, c * w.l_x, w.l_x, 1, l_l)
        assert np.abs(out[sl] - ref).max() < TOL["bf16"], c
        one = host(r.encode_chunk(dq[sl], dk, dv, c * w.l_x, w.l_x, 1, l_l))
        assert np.abs(one - ref).max() < TOL["bf16"], ("single", c)


@pytest.mark.parametrize("q_scale", [8.0, 32.0])
def test_qa_and_decode_when_the_softmax_maximum_keeps_rising(q_scale):
    w = W.C1.scaled(n_frames=8, n_q_tokens=20, name="C1-rising-qa")
    nf = w.tokens_per_frame
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    qq, qk, qv = W.question_qkv(w, 0)
    rng = np.random.default_rng(10)
    u = rng.standard_normal((w.n_kv_heads, w.head_dim))
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    k = W.round_to_bf16(k + 0.3 * np.arange(k.shape[0])[:, None, None] * u[None])
    qk = W.round_to_bf16(qk + (0.3 * k.shape[0] + 10.0 * np.arange(w.n_q_tokens))[:, None, None] * u[None])
    qq = W.round_to_bf16(q_scale * (qq + np.repeat(u, w.group, axis=0)[None]))
    r = Rekv.for_workload(w)
    out = host(r.qa_attention(dev(qq, w)[None], dev(k, w)[None], dev(v, w)[None], dev(qk, w)[None], dev(qv, w)[None]))[0]
    ref = O.qa_attention(qq, k, v, qk, qv)
    assert np.abs(out - ref).max() < TOL["bf16"]
    one = host(r.decode_attention(dev(qq[-1:], w)[None], dev(k, w)[None], dev(v, w)[None], dev(qk, w)[None],
                                  dev(qv, w)[None], w.n_q_tokens))[0]
    assert np.abs(one - ref[-1:]).max() < TOL["bf16"]


# ----------------------------------------------------------------------------------------
# multi-chunk launches at benchmark shapes, against the oracle
# ----------------------------------------------------------------------------------------
def test_c3_shaped_launch_of_eight_chunks():
    """Eight chunks of four frames (784 tokens, 43 row blocks of 128 per KV head) behind a full
    window of 32 frames, in one launch - the launch shape the 28-layer configuration is timed in."""
    w = W.C3.scaled(n_frames=64, n_layers=1, name="C3-8chunks")
    nf, lx = w.tokens_per_frame, w.l_x
    q = W.frames_q(w, 32, 64)
    k, v = W.frames_k(w, 0, 64), W.frames_v(w, 0, 64)
    r = Rekv.for_workload(w)
    out = host(r.encode_chunk(dev(q, w), dev(k, w), dev(v, w), 32 * nf, lx, 8, w.l_l))
    for c in (0, 3, 7):
        sl = slice(c * lx, (c + 1) * lx)
        ref = O.encode_chunks(q[sl], k, v, 32 * nf + c * lx, lx, 1, w.l_l)
        assert np.abs(out[sl] - ref).max() < TOL["bf16"], c


def test_c4_shaped_launch_of_eight_chunks():
    """Eight one-frame chunks at the 72B-class head layout (64 query heads, 8 KV heads) behind a
    full window of 16 frames, in one launch."""
    w = W.C4.scaled(n_frames=24, name="C4-8chunks")
    nf = w.tokens_per_frame
    q = W.frames_q(w, 16, 24)
    k, v = W.frames_k(w, 0, 24), W.frames_v(w, 0, 24)
    r = Rekv.for_workload(w)
    out = host(r.encode_chunk(dev(q, w), dev(k, w), dev(v, w), 16 * nf, nf, 8, w.l_l))
    for c in (0, 5, 7):
        sl = slice(c * nf, (c + 1) * nf)
        ref = O.encode_chunks(q[sl], k, v, (16 + c) * nf, nf, 1, w.l_l)
        assert np.abs(out[sl] - ref).max() < TOL["bf16"], c


# ----------------------------------------------------------------------------------------
# side stream ordering: the gather from host memory and the offload wait for the caller's stream
# ----------------------------------------------------------------------------------------
def _long_kernel(r, ms_target=40):
    """Queues a matrix-core probe launch of roughly ms_target milliseconds on the current stream."""
    sink = torch.empty(2048 * 256, dtype=torch.float32, device=DEV)
    r.probe_mfma(sink, 2048, 20000 * ms_target // 6)        # 2048 x 20000 iterations take about 6 ms
    return sink


@pytest.mark.parametrize("host_mode", [1, 2])
def test_host_gather_waits_for_work_queued_before_it(host_mode):
    """The index list is written on the caller's stream behind a long kernel; the gather from pinned
    host memory runs on the library's side stream and must still see that list, and the QA
    attention queued after it must see the gathered data."""
    w = W.C1.scaled(n_frames=12)
    nf = w.tokens_per_frame
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    tdt = torch.bfloat16
    hk = torch.from_numpy(np.ascontiguousarray(k)).to(tdt).pin_memory()
    hv = torch.from_numpy(np.ascontiguousarray(v)).to(tdt).pin_memory()
    r = Rekv.for_workload(w)
    sel = torch.tensor([[1, 4, 5, 9]], dtype=torch.int32, device=DEV)
    idx = torch.full((1, 4), -1, dtype=torch.int32, device=DEV)
    gk = torch.zeros((1, 4 * nf, w.n_kv_heads, w.head_dim), dtype=tdt, device=DEV)
    gv = torch.zeros_like(gk)
    qq, qk, qv = W.question_qkv(w, 0)
    dq, dqk, dqv = dev(qq, w)[None], dev(qk, w)[None], dev(qv, w)[None]
    torch.cuda.synchronize()
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)
    t0.record()
    sink = _long_kernel(r)
    t1.record()
    idx.copy_(sel)                                           # queued behind the long kernel
    r.gather_kv(hk, hv, idx, n_src_frames=w.n_frames, dst_k=gk, dst_v=gv, host_mode=host_mode)
    out = r.qa_attention(dq, gk, gv, dqk, dqv)
    torch.cuda.synchronize()
    assert t0.elapsed_time(t1) > 5.0                         # the kernel ahead really was long
    rk, rv = O.gather_kv(k, v, [1, 4, 5, 9], nf)
    assert host(gk)[0].tobytes() == rk.astype(np.float64).tobytes()
    assert host(gv)[0].tobytes() == rv.astype(np.float64).tobytes()
    assert np.abs(host(out)[0] - O.qa_attention(qq, rk, rv, qk, qv)).max() < TOL["bf16"]
    assert torch.isfinite(sink).all()


def test_offload_waits_for_the_kernel_that_writes_the_kv():
    """K/V are written on the caller's stream behind a long kernel; the offload copies on the side
    stream must carry the written values, not what the buffers held before."""
    w = W.C1.scaled(n_frames=6)
    nf = w.tokens_per_frame
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    src_k, src_v = dev(k, w), dev(v, w)
    dk, dv = torch.zeros_like(src_k), torch.zeros_like(src_v)
    hk = torch.zeros(src_k.shape, dtype=torch.bfloat16).pin_memory()
    hv = torch.zeros(src_v.shape, dtype=torch.bfloat16).pin_memory()
    r = Rekv.for_workload(w)
    torch.cuda.synchronize()
    _long_kernel(r)
    dk.copy_(src_k)
    dv.copy_(src_v)
    r.offload_kv(dk, dv, hk, hv, 1, 4)
    r.offload_wait()
    sl = slice(1 * nf, 5 * nf)
    assert torch.equal(hk[sl], src_k[sl].cpu()) and torch.equal(hv[sl], src_v[sl].cpu())
    assert not hk[:nf].any() and not hk[5 * nf:].any()      # frames outside the range were not touched
    torch.cuda.synchronize()


def test_offload_join_orders_later_writes_behind_the_copies():
    """The slots of offloaded frames are overwritten on the caller's stream right after
    rekv_offload_join, with no host wait in between: the host copies must hold the original
    values.  The buffers are large enough (37 MB each) that the copies are still running when
    the overwrite is queued."""
    w = W.C1.scaled(n_frames=96)
    nf = w.tokens_per_frame
    shape = (w.n_frames * nf, w.n_kv_heads, w.head_dim)
    g = torch.Generator(device=DEV).manual_seed(31)
    dk = torch.randn(shape, device=DEV, generator=g).to(torch.bfloat16)
    dv = torch.randn(shape, device=DEV, generator=g).to(torch.bfloat16)
    keep_k, keep_v = dk.clone(), dv.clone()
    hk = torch.zeros(shape, dtype=torch.bfloat16).pin_memory()
    hv = torch.zeros(shape, dtype=torch.bfloat16).pin_memory()
    r = Rekv.for_workload(w)
    torch.cuda.synchronize()
    r.offload_kv(dk, dv, hk, hv, 0, w.n_frames)
    r.offload_join()
    dk.fill_(7.0)                      # queued behind the join on the caller's stream
    dv.fill_(-7.0)
    r.offload_wait()
    torch.cuda.synchronize()
    assert torch.equal(hk, keep_k.cpu()) and torch.equal(hv, keep_v.cpu())
    assert bool((dk == 7.0).all()) and bool((dv == -7.0).all())


# ----------------------------------------------------------------------------------------
# per-layer gather in one launch
# ----------------------------------------------------------------------------------------
def test_gather_of_several_layers_in_one_launch():
    """Three layers, each with its own K/V arenas and its own selection (one with -1 padding):
    bit-equal to the oracle's gather layer by layer and to one rekv_gather_kv call per layer."""
    w = W.C3.scaled(n_frames=20, n_layers=3, name="C3-gather")
    nf = w.tokens_per_frame
    r = Rekv.for_workload(w)
    rng = np.random.default_rng(21)
    ks = [W.frames_k(w, 0, w.n_frames, layer) for layer in range(3)]
    vs = [W.frames_v(w, 0, w.n_frames, layer) for layer in range(3)]
    dks, dvs = [dev(x, w) for x in ks], [dev(x, w) for x in vs]
    nq, k = 2, 5
    idx = np.stack([np.stack([np.sort(rng.choice(w.n_frames, size=k, replace=False)) for _ in range(nq)]) for _ in range(3)]).astype(np.int32)
    idx[1, 0, 3:] = -1
    didx = torch.from_numpy(idx).to(DEV)
    gk, gv = r.gather_kv_layers(dks, dvs, didx, n_src_frames=w.n_frames)
    assert gk.shape == (3, nq, k * nf, w.n_kv_heads, w.head_dim)
    for layer in range(3):
        one_k, one_v = r.gather_kv(dks[layer], dvs[layer], didx[layer], n_src_frames=w.n_frames)
        assert torch.equal(gk[layer], one_k) and torch.equal(gv[layer], one_v)
        for q in range(nq):
            sel = [f for f in idx[layer, q] if f >= 0]
            rk, rv = O.gather_kv(ks[layer], vs[layer], sel, nf)
            n = len(sel) * nf
            assert host(gk)[layer, q, :n].tobytes() == rk.astype(np.float64).tobytes()
            assert host(gv)[layer, q, :n].tobytes() == rv.astype(np.float64).tobytes()
            assert not host(gk)[layer, q, n:].any()


# ----------------------------------------------------------------------------------------
# position policy of the retrieved keys on the gather-free path and for offloaded KV
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("w0,mode,src_rotated,layout", [
    (W.C1, "consecutive", False, "half"), (W.C1, "static", True, "half"), (W.C4, "consecutive", True, "interleaved"),
    (W.C0.scaled(tokens_per_frame=7, n_q_heads=4, n_kv_heads=2, name="C0p"), "consecutive", True, "half"),
    (W.C1.scaled(n_q_heads=14, n_kv_heads=2, head_dim=64, name="C1-0.5B"), "consecutive", True, "half")],
    ids=["7B-plain-cache", "7B-static", "72B-interleaved", "f32", "0.5B-D64"])
def test_in_place_attention_with_repositioned_keys(w0, mode, src_rotated, layout):
    """Values read in place through the frame list, keys turned to consecutive (or one static)
    position by the pre-pass: against the oracle's gather-with-positions followed by Eq. 3.  The
    second question's selection is shorter than the list (n_sel)."""
    w = w0.scaled(n_frames=24, n_q_tokens=11)
    nf = w.tokens_per_frame
    r = Rekv.for_workload(w)
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    src_off = 700_000
    if src_rotated:
        k = O.apply_rope(k, src_off + np.arange(k.shape[0]), layout=layout)
        k = W.round_to_bf16(k) if w.dtype == "bf16" else k.astype(np.float32).astype(np.float64)
    idx = np.array([[2, 5, 6, 11, 20], [0, 9, 23, -1, -1]], dtype=np.int32)
    n_sel = torch.tensor([5, 3], dtype=torch.int32, device=DEV)
    qs = [W.question_qkv(w, i) for i in range(2)]
    dq, dqk, dqv = (dev(np.stack([x[j] for x in qs]), w) for j in range(3))
    out, k_pos = r.attention_indexed_rope(dq, dev(k, w), dev(v, w), torch.from_numpy(idx).to(DEV), dqk, dqv, w.n_q_tokens,
                                          n_src_frames=w.n_frames, n_sel=n_sel, mode=mode, pos_offset=35,
                                          src_rotated=src_rotated, src_pos_offset=src_off, layout=layout)
    out = host(out)
    for i in range(2):
        frames = [f for f in idx[i] if f >= 0]
        rk, rv = O.gather_kv_rope(k, v, frames, nf, mode=mode, pos_offset=35, src_rotated=src_rotated,
                                  src_pos_offset=src_off, layout=layout)
        # the oracle's keys, rounded once to the storage type as the pre-pass stores them
        rk = W.round_to_bf16(rk) if w.dtype == "bf16" else rk.astype(np.float32).astype(np.float64)
        ref = O.decode_attention(qs[i][0], rk, rv, qs[i][1], qs[i][2])
        err = np.abs(out[i] - ref).max()
        assert err < TOL[w.dtype], (i, err)
    # the same through gather-with-positions + attention of this library
    gk, gv = r.gather_kv_rope(dev(k, w), dev(v, w), torch.from_numpy(idx).to(DEV), n_src_frames=w.n_frames, mode=mode,
                              pos_offset=35, src_rotated=src_rotated, src_pos_offset=src_off, layout=layout)
    assert torch.equal(gk, k_pos)
    via_gather = host(r.decode_attention(dq, gk, gv, dqk, dqv, w.n_q_tokens, n_sel=n_sel))
    assert np.abs(via_gather - out).max() < 1e-6 + (4e-3 if w.dtype == "bf16" else 0)


def test_position_policy_on_offloaded_kv():
    """The gather with positions reading pinned host arenas (offloaded KV): bit-equal to the same
    call on HBM arenas."""
    w = W.C1.scaled(n_frames=20)
    k, v = W.frames_k(w, 0, w.n_frames), W.frames_v(w, 0, w.n_frames)
    r = Rekv.for_workload(w)
    dk, dv = dev(k, w), dev(v, w)
    hk, hv = dk.cpu().pin_memory(), dv.cpu().pin_memory()
    idx = torch.tensor([[17, 3, 4, 9, -1], [0, 19, 18, -1, -1]], dtype=torch.int32, device=DEV)
    a = r.gather_kv_rope(dk, dv, idx, mode="consecutive", pos_offset=35)
    b = r.gather_kv_rope(hk, hv, idx, mode="consecutive", pos_offset=35)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
