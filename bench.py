"""Benchmark of the ReKV hot path on one MI355X.

A step is one pass of the whole path over one stream of synthetic video tokens and one
question: sliding-window encode of every chunk (one multi-chunk launch), the frame vectors,
retrieval (pool + cosine + top-k), the KV gather and the QA attention.  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C0..C4] [--no-cpu-baseline]
                    [--no-extras]

After the timed steps the default run also reports, outside `value`: the same stream encoded one
launch per chunk (`streaming_tokens_per_s`), the encode launch on all-zero inputs (what the data's
switching activity costs in sustained clock), the bandwidth-bound kernels at the 72B-class shapes of
C4 (`hbm_kernels`: their tables are too small at C1 to say anything about HBM), the box's own copy
and MFMA-loop rates, and the CPU oracle on a bounded sample.  `--no-extras` leaves the first three out.

The default workload is C1, the configuration the metric is quoted on; C2 (hour-long stream, KV
offloaded to pinned host memory), C3 (28 layers) and C4 (64 concurrent questions) run the same
step at their shapes, for the bandwidth-bound kernels' HBM fractions.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP32_VALU_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

TRAFFIC_PROFILE = {"C1-7B-1layer": "profiles/attn_bf16_encode_C1_hbm_traffic.txt"}
ENCODE_KERNEL_SOURCE = "paper_2503_00540_amd/csrc/attention_bf16.hip"


def measured_traffic(workload_name):
    """HBM bytes of one encode launch as the committed rocprofv3 counter summary states them
    (FETCH_SIZE and WRITE_SIZE, calibrated on the probe copy of the same runs; written by
    paper_2503_00540_amd/profile_summary.py).  A counter run cannot happen inside this process, so
    the value is quoted with its source, and only while the kernel source it was measured on is
    the one in the tree; otherwise null."""
    import hashlib
    import re
    rel = TRAFFIC_PROFILE.get(workload_name)
    if not rel or not os.path.exists(os.path.join(ROOT, rel)):
        return None, "no counter summary for this workload under profiles/"
    text = open(os.path.join(ROOT, rel)).read()
    m = re.search(r"^traffic_bytes_per_launch: (\d+)$", text, re.M)
    h = re.search(r"^kernel_source_sha256: ([0-9a-f]+)$", text, re.M)
    if not m or not h:
        return None, f"{rel} carries no machine-readable traffic line"
    sha = hashlib.sha256(open(os.path.join(ROOT, ENCODE_KERNEL_SOURCE), "rb").read()).hexdigest()
    if sha != h.group(1):
        return None, f"{rel} was measured on another version of {ENCODE_KERNEL_SOURCE}"
    return int(m.group(1)), f"{rel} (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this command, same kernel source)"


def encode_flops(w) -> float:
    """Algorithmic FLOP of one encode pass over the stream: 4*D*Hq per visible (q, k) pair."""
    n_chunks = w.n_frames // w.chunk_frames
    pairs = 0
    for c in range(n_chunks):
        win = min(w.l_l, c * w.l_x)
        pairs += w.l_x * win + w.l_x * (w.l_x + 1) // 2
    return 4.0 * w.head_dim * w.n_q_heads * pairs


def qa_flops(w) -> float:
    return 4.0 * w.head_dim * w.n_q_heads * w.n_questions * (
        w.n_q_tokens * w.top_k * w.tokens_per_frame + w.n_q_tokens * (w.n_q_tokens + 1) // 2)


def cpu_baseline(w, seconds_target=12.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: steady-state
    chunks of the encode (batches of 16 until about `seconds_target` seconds have been spent),
    then the frame vectors, one retrieval, the gather and one QA pass over the sampled frames."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import rekv_oracle as O
    from paper_2503_00540_amd import workloads as W

    n_chunks = w.n_frames // w.chunk_frames
    win_chunks = -(-w.window_frames // w.chunk_frames)
    c0 = min(win_chunks, n_chunks - 1)                   # first steady-state chunk
    batch = 16 if w.dtype == "bf16" else n_chunks
    done, t_enc = 0, 0.0
    k = v = None
    while c0 + done < n_chunks and t_enc < seconds_target:
        c_lo, c_hi = c0 + done, min(c0 + done + batch, n_chunks)
        f0, f1 = max(0, c_lo * w.chunk_frames - w.window_frames), c_hi * w.chunk_frames
        k, v = W.frames_k(w, f0, f1), W.frames_v(w, f0, f1)
        q = W.frames_q(w, c_lo * w.chunk_frames, f1)
        t = time.perf_counter()
        O.encode_chunks(q, k, v, (c_lo * w.chunk_frames - f0) * w.tokens_per_frame, w.l_x, c_hi - c_lo, w.l_l)
        t_enc += time.perf_counter() - t
        done += c_hi - c_lo
    n_vis = k.shape[0] // w.tokens_per_frame
    qq, qk, qv = W.question_qkv(w, 0, n_visible=n_vis)
    t = time.perf_counter()
    fk = O.frame_keys(k, n_vis, w.tokens_per_frame)
    idx, _ = O.retrieve(fk, qq, w.n_kv_heads, min(w.top_k, n_vis))
    rk, rv = O.gather_kv(k, v, idx, w.tokens_per_frame)
    O.qa_attention(qq, rk, rv, qk, qv)
    t_qa = time.perf_counter() - t
    threads = max([i["num_threads"] for i in threadpool_info()] + [1])
    tokens = done * w.l_x
    return {"value": tokens / (t_enc + t_qa), "unit": "video tokens/s", "cores": threads, "kind": "oracle",
            "cores_means": "threads of the BLAS library behind numpy's fp64 matrix products; the oracle's own "
                           "loops over heads and chunks are serial Python",
            "sample": f"{done} steady-state chunks of {w.l_x} tokens (window {w.l_l}) encoded in "
                      f"{t_enc:.2f} s, plus frame vectors, one retrieval, gather and one QA pass over "
                      f"{n_vis} frames in {t_qa:.3f} s; fp64 numpy (BLAS threads = cores)",
            "encode_s": t_enc, "retrieval_qa_s": t_qa}


def host_inputs(w, torch, np):
    """C0 / C1: the seeded host generator of workloads.py (the arrays the parity tests use)."""
    from paper_2503_00540_amd import workloads as W
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32

    def dev(x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(tdt).to("cuda:0")

    def cat(fn):
        return torch.cat([dev(fn(w, f, min(f + 64, w.n_frames))) for f in range(0, w.n_frames, 64)])

    qs = [W.question_qkv(w, i) for i in range(w.n_questions)]
    planted = [W.planted_frames(w, i).tolist() for i in range(w.n_questions)]
    return {"q": [cat(W.frames_q)], "k": [cat(W.frames_k)], "v": [cat(W.frames_v)],
            "qq": dev(np.stack([x[0] for x in qs])), "qk": dev(np.stack([x[1] for x in qs])),
            "qv": dev(np.stack([x[2] for x in qs])), "planted": planted}


def gpu_inputs(w, torch):
    """C2 / C3 / C4: the same recipe (N(0,1) + per-frame offset of sigma 0.5; question queries =
    planted frames' key offsets + N(0, 0.3^2)) drawn on the GPU with torch's seeded generator -
    these streams are too long to draw on the host within the run.  Q is kept for two layers
    and reused alternately; every layer has its own K/V, as it would in HBM."""
    g = torch.Generator(device="cuda:0").manual_seed(w.seed)
    gc = torch.Generator().manual_seed(w.seed)
    F, nf, G = w.n_frames, w.tokens_per_frame, w.group

    def stream(heads):
        out = torch.empty((F * nf, heads, w.head_dim), dtype=torch.bfloat16, device="cuda:0")
        off = 0.5 * torch.randn((F, 1, heads, w.head_dim), device="cuda:0", generator=g)
        for f in range(0, F, 128):
            f1 = min(f + 128, F)
            x = torch.randn((f1 - f, nf, heads, w.head_dim), device="cuda:0", generator=g) + off[f:f1]
            out[f * nf:f1 * nf] = x.reshape(-1, heads, w.head_dim).to(torch.bfloat16)
        return out, off[:, 0]

    d = {"q": [stream(w.n_q_heads)[0] for _ in range(min(2, w.n_layers))], "k": [], "v": [],
         "qq": [], "qk": [], "qv": [], "planted": []}
    for layer in range(w.n_layers):
        k, off_k = stream(w.n_kv_heads)
        d["k"].append(k)
        d["v"].append(stream(w.n_kv_heads)[0])
        for _ in range(w.n_questions):
            p = torch.randperm(F, generator=gc)[:w.n_planted].sort().values
            d["planted"].append(p.tolist())
            base = off_k[p.to("cuda:0")][torch.arange(w.n_q_tokens, device="cuda:0") % w.n_planted]   # [N_q, Hkv, D]
            qq = base.repeat_interleave(G, dim=1) + 0.3 * torch.randn((w.n_q_tokens, w.n_q_heads, w.head_dim),
                                                                      device="cuda:0", generator=g)
            d["qq"].append(qq.to(torch.bfloat16))
            d["qk"].append(torch.randn((w.n_q_tokens, w.n_kv_heads, w.head_dim), device="cuda:0", generator=g).to(torch.bfloat16))
            d["qv"].append(torch.randn((w.n_q_tokens, w.n_kv_heads, w.head_dim), device="cuda:0", generator=g).to(torch.bfloat16))
    for key in ("qq", "qk", "qv"):
        d[key] = torch.stack(d[key])
    return d


PROBE_COPY_BYTES = 1 << 30


def box_peaks(r, torch, copy_only=False):
    """What this GPU sustains: a plain streaming copy (bytes read + written per second) and a
    register-resident bf16 MFMA loop.  Context for the roofline fractions, which stay priced
    against the published peaks."""
    src = torch.empty(PROBE_COPY_BYTES, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    t_copy = timed(lambda: r.probe_copy(dst, src), 5)
    out = {"copy_bytes": PROBE_COPY_BYTES, "copy_read_plus_write_GBs": 2 * PROBE_COPY_BYTES / t_copy / 1e9}
    if not copy_only:
        n_wg, n_it = 2048, 20000
        sink = torch.empty(n_wg * 256, dtype=torch.float32, device="cuda:0")
        flop = [0.0]

        def mf():
            flop[0] = r.probe_mfma(sink, n_wg, n_it)
        t_mfma = timed(mf, 3)
        out["mfma_bf16_loop_TFLOPs"] = flop[0] / t_mfma / 1e12
    return out


def hbm_kernels_at_c4_shapes(torch, timed_us):
    """The bandwidth-bound kernels at the 72B-class shapes of C4 (64 questions on a 2,048-frame
    stream; random data of the benchmark's distribution drawn on the GPU): frame vectors over the
    stream's keys, batched retrieval, the gather of 64 x 32 frames and one decode step over the
    gathered KV.  Algorithmic bytes, HIP-event time per call, fraction of the 8 TB/s HBM peak."""
    from paper_2503_00540_amd import workloads as W
    from paper_2503_00540_amd.rekv import Rekv
    w = W.C4
    r = Rekv.for_workload(w)
    g = torch.Generator(device="cuda:0").manual_seed(w.seed)
    F, nf, nq, dp = w.n_frames, w.tokens_per_frame, w.n_questions, w.d_prime

    def stream():
        out = torch.empty((F * nf, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16, device="cuda:0")
        for f in range(0, F, 256):
            off = 0.5 * torch.randn((256, 1, w.n_kv_heads, w.head_dim), device="cuda:0", generator=g)
            x = torch.randn((256, nf, w.n_kv_heads, w.head_dim), device="cuda:0", generator=g) + off
            out[f * nf:(f + 256) * nf] = x.reshape(-1, w.n_kv_heads, w.head_dim).to(torch.bfloat16)
        return out

    k, v = stream(), stream()
    fk = torch.empty((F, dp), dtype=torch.float32, device="cuda:0")
    qq = torch.randn((nq, w.n_q_tokens, w.n_q_heads, w.head_dim), device="cuda:0", generator=g).to(torch.bfloat16)
    gk = torch.empty((nq, w.top_k * nf, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16, device="cuda:0")
    gv = torch.empty_like(gk)
    n_text = w.n_q_tokens + 64
    kt = torch.randn((nq, n_text, w.n_kv_heads, w.head_dim), device="cuda:0", generator=g).to(torch.bfloat16)
    vt = torch.randn((nq, n_text, w.n_kv_heads, w.head_dim), device="cuda:0", generator=g).to(torch.bfloat16)
    q1 = torch.randn((nq, 1, w.n_q_heads, w.head_dim), device="cuda:0", generator=g).to(torch.bfloat16)
    o1 = torch.empty_like(q1)
    r.frame_keys(k, F, out=fk)
    idx, _, _ = r.retrieve_topk(fk, F, qq, w.top_k)
    rows = {
        "frame_keys": (F * nf * dp * 2 + F * dp * 4, lambda: r.frame_keys(k, F, out=fk)),
        "retrieve_pool_score_topk": (nq * w.n_q_tokens * w.n_q_heads * w.head_dim * 2 + F * dp * 4 + nq * F * 4 * 2,
                                     lambda: r.retrieve_topk(fk, F, qq, w.top_k)),
        "gather": (2 * 2 * nq * w.top_k * nf * dp * 2, lambda: r.gather_kv(k, v, idx, n_src_frames=F, dst_k=gk, dst_v=gv)),
        "decode_step": (2 * nq * (w.top_k * nf + n_text) * dp * 2, lambda: r.decode_attention(q1, gk, gv, kt, vt, n_text, out=o1)),
    }
    out = {"shapes": f"{w.name}: {F} frames x {nf} tokens, Hq/Hkv/D {w.n_q_heads}/{w.n_kv_heads}/{w.head_dim}, "
                     f"{nq} questions, top-k {w.top_k}; HIP-event time per call over 20 calls back to back",
           "peak_GBs": PEAK_HBM_GBS}
    for name, (nbytes, fn) in rows.items():
        us = timed_us(fn)
        out[name] = {"bytes": nbytes, "us": us, "GBs": nbytes / us / 1e3, "frac_of_hbm_peak": nbytes / us / 1e3 / PEAK_HBM_GBS}
    out["retrieve_pool_score_topk"]["note"] = ("three dependent launches of a few us each; the bytes are the questions' "
                                               "queries, the frame table once and the scores written and read")
    return out


def host_link_peak(torch, n_bytes):
    """One pinned-host-to-HBM copy of n_bytes through the copy engine: the rate the gather from
    offloaded KV is to be read against."""
    src = torch.empty(n_bytes, dtype=torch.uint8, pin_memory=True)
    src.fill_(1)
    dst = torch.empty(n_bytes, dtype=torch.uint8, device="cuda:0")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    dst.copy_(src, non_blocking=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        dst.copy_(src, non_blocking=True)
    e1.record()
    torch.cuda.synchronize()
    return 5 * n_bytes / (e0.elapsed_time(e1) * 1e-3) / 1e9


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="C1", choices=["C0", "C1", "C2", "C3", "C4"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="leave out the measurements after the timed steps that launch further kernels: the stream "
                         "encoded one launch per chunk, the encode launch on all-zero inputs, the C4-shaped "
                         "bandwidth-bound kernels")
    ap.add_argument("--probe-copy-only", action="store_true",
                    help="run only the known-size copy kernel (the calibration run of the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU by design (one MI355X runs the whole path); "
                 "run with --gpus 1")

    import numpy as np
    import torch

    from paper_2503_00540_amd import workloads as W
    from paper_2503_00540_amd.rekv import Rekv

    w = W.CONFIGS[args.workload]
    big = args.workload in ("C2", "C3", "C4")
    steps = args.steps if args.steps is not None else (3 if big else 20)
    warmup = args.warmup if args.warmup is not None else (1 if big else 3)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    torch.cuda.set_device(0)
    r = Rekv.for_workload(w)
    if args.probe_copy_only:
        print(json.dumps({"box_peaks": box_peaks(r, torch, copy_only=True)}))
        return
    d = gpu_inputs(w, torch) if big else host_inputs(w, torch, np)     # resident in HBM before timing

    L, nq, F, nf = w.n_layers, w.n_questions, w.n_frames, w.tokens_per_frame
    n_chunks = F // w.chunk_frames
    d_prime = w.d_prime
    out = torch.empty_like(d["q"][0])
    fk = torch.empty((L, F, d_prime), dtype=torch.float32, device="cuda:0")
    ret_shape = (L * nq, w.top_k * nf, w.n_kv_heads, w.head_dim)
    gk, gv = torch.empty(ret_shape, dtype=tdt, device="cuda:0"), torch.empty(ret_shape, dtype=tdt, device="cuda:0")
    qa_out = torch.empty_like(d["qq"])
    hk = hv = None
    if w.kv_on_host:
        hk = torch.empty(d["k"][0].shape, dtype=tdt, pin_memory=True)
        hv = torch.empty(d["v"][0].shape, dtype=tdt, pin_memory=True)

    names = ["encode", "frame_keys", "offload_issue", "offload_wait", "retrieve", "gather", "qa"]
    N_SEG = 8

    def one_step(log=None):
        def rec(name):
            if log is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                log.append((name, e))
        for layer in range(L):
            if w.kv_on_host:
                # the stream is encoded in N_SEG launches; each segment's KV leaves HBM on the side
                # stream (copy engine) while the next segment is being encoded
                q_l, k_l, v_l = d["q"][layer % len(d["q"])], d["k"][layer], d["v"][layer]
                for sgm in range(N_SEG):
                    c0, c1 = sgm * n_chunks // N_SEG, (sgm + 1) * n_chunks // N_SEG
                    rec("encode")
                    r.encode_chunk(q_l[c0 * w.l_x:c1 * w.l_x], k_l, v_l, c0 * w.l_x, w.l_x, c1 - c0, w.l_l,
                                   out=out[c0 * w.l_x:c1 * w.l_x])
                    rec("frame_keys")
                    f0, f1 = c0 * w.chunk_frames, c1 * w.chunk_frames
                    r.frame_keys(k_l[f0 * nf:f1 * nf], f1 - f0, out=fk[layer][f0:f1])
                    rec("offload_issue")
                    r.offload_kv(k_l, v_l, hk, hv, f0, f1 - f0)
                continue
            rec("encode")
            r.encode_chunk(d["q"][layer % len(d["q"])], d["k"][layer], d["v"][layer], 0, w.l_x, n_chunks, w.l_l, out=out)
            rec("frame_keys")
            r.frame_keys(d["k"][layer], F, out=fk[layer])
        if w.kv_on_host:               # the question arrives once the stream's KV has left HBM
            rec("offload_wait")
            r.offload_wait()
        rec("retrieve")
        idx, n_sel, _ = r.retrieve_topk(fk, F, d["qq"], w.top_k, frame_keys_stride=F * d_prime if L > 1 else 0)
        rec("gather")
        if w.kv_on_host:
            r.gather_kv(hk, hv, idx, n_src_frames=F, dst_k=gk, dst_v=gv)
        elif L > 1:                    # every layer's selection from its own arenas, one launch
            r.gather_kv_layers(d["k"], d["v"], idx.view(L, nq, w.top_k), n_src_frames=F, dst_k=gk, dst_v=gv)
        else:
            r.gather_kv(d["k"][0], d["v"][0], idx, n_src_frames=F, dst_k=gk, dst_v=gv)
        rec("qa")
        r.qa_attention(d["qq"], gk, gv, d["qk"], d["qv"], out=qa_out, n_sel=n_sel)
        rec(None)
        return idx

    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()
    logs = [[] for _ in range(steps)]
    t0 = time.perf_counter()
    for s in range(steps):
        idx = one_step(logs[s])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms = {n: 0.0 for n in names}
    for log in logs:
        for (name, e0), (_, e1) in zip(log[:-1], log[1:]):
            ms[name] += e0.elapsed_time(e1) / steps
    # per-step latency from "question available" to "QA output ready" (retrieve + gather + QA)
    lat = []
    for log in logs:
        t = 0.0
        for (name, e0), (_, e1) in zip(log[:-1], log[1:]):
            if name in ("retrieve", "gather", "qa"):
                t += e0.elapsed_time(e1)
        lat.append(t)
    lat.sort()
    ms_per_step = elapsed / steps * 1e3
    n_tokens = L * w.n_tokens
    tokens_per_s = n_tokens / (elapsed / steps)

    # the same stream encoded chunk by chunk (one launch per chunk, as a live stream arrives)
    streaming_s = None
    extras = not args.no_extras
    if extras:
        dq, dk, dv = d["q"][0], d["k"][0], d["v"][0]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for c in range(n_chunks):
            r.encode_chunk(dq[c * w.l_x:(c + 1) * w.l_x], dk, dv, c * w.l_x, w.l_x, 1, w.l_l,
                           out=out[c * w.l_x:(c + 1) * w.l_x])
        torch.cuda.synchronize()
        streaming_s = time.perf_counter() - t1

    # beyond the step: one decode-step attention over the retrieved KV (Eq. 3, X = the current
    # token, 64 tokens already generated) and block-level retrieval at b = 8, timed on their own
    def timed_us(fn, reps=20):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    n_text = w.n_q_tokens + 64
    g = torch.Generator(device="cuda:0").manual_seed(7)
    kt = torch.randn((nq, 256, w.n_kv_heads, w.head_dim), device="cuda:0", generator=g).to(tdt)
    vt = torch.randn((nq, 256, w.n_kv_heads, w.head_dim), device="cuda:0", generator=g).to(tdt)
    q1 = torch.randn((nq, 1, w.n_q_heads, w.head_dim), device="cuda:0", generator=g).to(tdt)
    o1 = torch.empty_like(q1)
    decode_us = timed_us(lambda: r.decode_attention(q1, gk[:nq], gv[:nq], kt, vt, n_text, out=o1))
    decode_bytes = 2 * nq * (w.top_k * nf + n_text) * d_prime * (2 if w.dtype == "bf16" else 4)
    # QA attention of layer 0 with the retrieved frames read in place (no gathered copy), against
    # gather + QA attention of the same questions
    idx0 = idx[:nq].contiguous()
    qa0 = torch.empty_like(d["qq"][:nq])
    indexed_us = gathered_us = None
    if not w.kv_on_host:
        indexed_us = timed_us(lambda: r.attention_indexed(d["qq"][:nq], d["k"][0], d["v"][0], idx0, w.top_k,
                                                           d["qk"][:nq], d["qv"][:nq], w.n_q_tokens,
                                                           n_src_frames=F, out=qa0))

        def gather_then_qa():
            r.gather_kv(d["k"][0], d["v"][0], idx0, n_src_frames=F, dst_k=gk[:nq], dst_v=gv[:nq])
            r.qa_attention(d["qq"][:nq], gk[:nq], gv[:nq], d["qk"][:nq], d["qv"][:nq], out=qa0)
        gathered_us = timed_us(gather_then_qa)
    b_blk = 8
    kb = -(-w.top_k // b_blk)
    bk = torch.empty((-(-F // b_blk), d_prime), dtype=torch.float32, device="cuda:0")
    qq0 = d["qq"][:nq]

    def block_retrieval():
        r.block_keys(fk[0], F, b_blk, out=bk)
        blk, _, _ = r.retrieve_topk(bk, bk.shape[0], qq0, kb)
        return r.expand_blocks(blk, b_blk, F)
    block_us = timed_us(block_retrieval)

    # the same encode launch on all-zero inputs: same instructions and traffic, least switching
    # power; the gap to the timed figure is what the data's toggling costs in sustained clock
    zero_tflops = None
    if w.dtype == "bf16" and extras:
        zq, zk = torch.zeros_like(d["q"][0]), torch.zeros_like(d["k"][0])
        zero_us = timed_us(lambda: r.encode_chunk(zq, zk, zk, 0, w.l_x, n_chunks, w.l_l, out=out), reps=5)
        zero_tflops = encode_flops(w) / zero_us / 1e6
        del zq, zk

    planted = [set(p) <= set(idx[i].tolist()) for i, p in enumerate(d["planted"])]
    fl = encode_flops(w)                                   # one launch = one layer's stream
    if w.dtype == "bf16":
        bound, peak = "mfma", PEAK_BF16_TFLOPS
    else:
        bound, peak = "alu", PEAK_FP32_VALU_TFLOPS
    n_launch = N_SEG if w.kv_on_host else 1                # encode launches per layer
    fl /= n_launch
    enc_launch_ms = ms["encode"] / (L * n_launch)
    achieved = fl / (enc_launch_ms * 1e-3) / 1e12
    es = 2 if w.dtype == "bf16" else 4
    gather_bytes = 2 * L * nq * w.top_k * nf * d_prime * es          # K and V, read once (and written once)
    fk_bytes = L * (w.n_tokens * d_prime * es + F * d_prime * 4)
    traffic, traffic_source = measured_traffic(w.name)
    result = {
        "metric": "video tokens/s encoded (windowed attn, MFMA %); retrieval+QA latency ms (HBM GB/s)",
        "value": tokens_per_s, "unit": "video tokens/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: {L} layer(s), {F} frames x {nf} tokens, "
                               f"Hq/Hkv/D {w.n_q_heads}/{w.n_kv_heads}/{w.head_dim}, chunk {w.l_x} tokens, "
                               f"window {w.l_l} tokens, {nq} question(s) of {w.n_q_tokens} tokens, "
                               f"top-k {w.top_k}, KV {'offloaded to pinned host memory' if w.kv_on_host else 'in HBM'}; "
                               f"a step = per layer: encode all {n_chunks} chunks in {N_SEG if w.kv_on_host else 1} launch(es) + frame vectors"
                               f"{' + KV offload' if w.kv_on_host else ''}; then retrieval + gather + QA attention",
                   "n_chunks_per_launch": n_chunks // (N_SEG if w.kv_on_host else 1)},
        "roofline": {"bound": bound, "kernel": "attn_bf16_kernel<D, true> (rekv_encode_chunk)" if w.dtype == "bf16"
                     else "attn_f32_kernel (rekv_encode_chunk)",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_flop_per_launch": fl, "avg_launch_ms": enc_launch_ms},
        "kernel_ms": ms,
        "retrieval_qa_latency_ms": ms["retrieve"] + ms["gather"] + ms["qa"],
        "retrieval_qa_latency_ms_median": lat[len(lat) // 2], "retrieval_qa_latency_ms_min": lat[0],
        "encode_only_tokens_per_s": n_tokens / (ms["encode"] * 1e-3),
        "streaming_tokens_per_s": w.n_tokens / streaming_s if streaming_s else None,
        "hbm": {("gather_host_link_GBs" if w.kv_on_host else "gather_read_plus_write_GBs"):
                (1 if w.kv_on_host else 2) * gather_bytes / (ms["gather"] * 1e-3) / 1e9,
                "frame_keys_GBs": fk_bytes / (ms["frame_keys"] * 1e-3) / 1e9,
                "retrieve_table_GBs": L * F * d_prime * 4 / (ms["retrieve"] * 1e-3) / 1e9,
                "qa_TFLOPs": L * qa_flops(w) / (ms["qa"] * 1e-3) / 1e12, "peak_GBs": PEAK_HBM_GBS},
        "planted_frames_retrieved": all(planted),
        "decode_step": {"us": decode_us, "kv_GBs": decode_bytes / decode_us / 1e3,
                        "what": f"{nq} question(s), 1 new token over {w.top_k * nf} retrieved + {n_text} text tokens, one layer"},
        "qa_indexed": {"us": indexed_us, "gather_plus_qa_us": gathered_us,
                       "what": "QA attention of one layer reading the retrieved frames in place vs gather + QA attention"},
        "block_retrieval": {"us": block_us, "b": b_blk, "blocks_selected": kb,
                            "what": "block vectors from the frame table + scores + top-k + frame list, one layer"},
        "box_peaks": dict(box_peaks(r, torch), encode_on_zero_inputs_TFLOPs=zero_tflops),
    }
    if streaming_s:
        result["streaming"] = {"launches": n_chunks, "wall_ms": streaming_s * 1e3, "us_per_chunk": streaming_s / n_chunks * 1e6,
                               "what": "the same stream encoded one rekv_encode_chunk call per chunk, back to back on one stream"}
    if w.kv_on_host:
        result["hbm"]["host_link_pinned_copy_GBs"] = host_link_peak(torch, gather_bytes)
        result["hbm"]["gather_frac_of_host_link"] = (result["hbm"]["gather_host_link_GBs"] /
                                                     result["hbm"]["host_link_pinned_copy_GBs"])
    if extras and w.dtype == "bf16":
        result["hbm_kernels"] = hbm_kernels_at_c4_shapes(torch, timed_us)
    bp = result["box_peaks"]
    if w.dtype == "bf16" and bp.get("mfma_bf16_loop_TFLOPs"):
        bp["encode_frac_of_mfma_loop"] = achieved / bp["mfma_bf16_loop_TFLOPs"]
    bp["gather_frac_of_copy"] = (None if w.kv_on_host else
                                 2 * gather_bytes / (ms["gather"] * 1e-3) / 1e9 / bp["copy_read_plus_write_GBs"])
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
