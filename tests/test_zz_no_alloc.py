"""The allocation-free decode entry point against the ordinary one: same kernels, static scratch
instead of the context's workspace.  Two calls in a row, the second with a smaller input.  Needs
a real MI355X."""
import numpy as np
import pytest
import torch

from oracle import rekv_oracle as O
from paper_2503_00540_amd import workloads as W
from paper_2503_00540_amd.rekv import Rekv, RekvError

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(w, nq, n_ret_frames, n_text, n_new, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    mk = lambda *s: torch.randn(*s, device=DEV, generator=g).to(tdt)
    nf = w.tokens_per_frame
    return (mk(nq, n_new, w.n_q_heads, w.head_dim), mk(nq, n_ret_frames * nf, w.n_kv_heads, w.head_dim),
            mk(nq, n_ret_frames * nf, w.n_kv_heads, w.head_dim), mk(nq, n_text + 3, w.n_kv_heads, w.head_dim),
            mk(nq, n_text + 3, w.n_kv_heads, w.head_dim))


@pytest.mark.parametrize("w", [W.C1, W.C0.scaled(tokens_per_frame=7, name="C0n")], ids=["bf16", "f32"])
def test_no_alloc_decode_equals_the_allocating_call(w):
    r = Rekv.for_workload(w)
    tol = 2e-2 if w.dtype == "bf16" else 1e-4
    # first call: one question, long retrieved context (key range split over many workgroups);
    # second call: smaller in every size, so it finds the first call's partial results in the scratch
    for nq, n_ret_frames, n_text, n_new, seed in ((1, 16, 96, 1, 1), (2, 3, 40, 2, 2)):
        q, kr, vr, kt, vt = _inputs(w, nq, n_ret_frames, n_text, n_new, seed)
        n_sel = torch.tensor([n_ret_frames] + [max(n_ret_frames - 1, 0)] * (nq - 1), dtype=torch.int32, device=DEV)
        ref = r.decode_attention(q, kr, vr, kt, vt, n_text, n_sel=n_sel)
        out = r.decode_attention(q, kr, vr, kt, vt, n_text, n_sel=n_sel, no_alloc=True)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), (out.float() - ref.float()).abs().max().item()
        # and both against the oracle, on the first question
        h = lambda t: t.detach().float().cpu().numpy().astype(np.float64)
        nv = int(n_sel[0]) * w.tokens_per_frame
        o_ref = O.decode_attention(h(q)[0], h(kr)[0, :nv], h(vr)[0, :nv], h(kt)[0, :n_text], h(vt)[0, :n_text])
        assert np.abs(h(out)[0] - o_ref).max() < tol


def test_no_alloc_decode_refuses_what_the_ordinary_call_refuses():
    w = W.C1
    r = Rekv.for_workload(w)
    q, kr, vr, kt, vt = _inputs(w, 1, 2, 20, 1, 3)
    with pytest.raises(RekvError):
        r.decode_attention(q, kr, vr, kt, vt, 0, no_alloc=True)            # fewer text rows than new tokens


def test_no_alloc_decode_captures_into_a_hip_graph_on_a_fresh_context():
    """What the entry point is for: a context that has never grown a workspace is captured into a HIP
    graph (the allocating call could not be: its first use allocates), and every replay, with eager
    library work and synchronisations in between, gives the eager result bit for bit."""
    w = W.C1
    q, kr, vr, kt, vt = _inputs(w, 1, 16, 96, 1, 5)          # split key range: the scratch is in use
    n_text = 96
    ref = Rekv.for_workload(w).decode_attention(q, kr, vr, kt, vt, n_text)      # another context
    fresh = Rekv.for_workload(w)
    out = torch.empty_like(q)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            fresh.decode_attention(q, kr, vr, kt, vt, n_text, out=out, no_alloc=True)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for _ in range(4):
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref)
        other = fresh.decode_attention(q, kr, vr, kt, vt, n_text, no_alloc=True)    # eager use of the same scratch
        torch.cuda.synchronize()
        assert torch.equal(other, ref)
