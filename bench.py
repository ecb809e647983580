"""Benchmark of the ReKV hot path on one MI355X.

A step is one pass of the whole path over one stream of synthetic video tokens and one
question: sliding-window encode of every chunk (one multi-chunk launch), the frame vectors,
retrieval (pool + cosine + top-k), the KV gather and the QA attention.  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C1] [--no-cpu-baseline]
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

# HBM traffic of one encode launch at C1 from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (see profiles/); None until measured for the workload.
MEASURED_TRAFFIC_BYTES = {}


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
            "sample": f"{done} steady-state chunks of {w.l_x} tokens (window {w.l_l}) encoded in "
                      f"{t_enc:.2f} s, plus frame vectors, one retrieval, gather and one QA pass over "
                      f"{n_vis} frames in {t_qa:.3f} s; fp64 numpy (BLAS threads = cores)",
            "encode_s": t_enc, "retrieval_qa_s": t_qa}


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU by design (one MI355X runs the whole path); "
                 "run with --gpus 1")

    import numpy as np
    import torch

    from paper_2503_00540_amd import workloads as W
    from paper_2503_00540_amd.rekv import Rekv

    w = W.CONFIGS[args.workload]
    if w.n_layers != 1 or w.kv_on_host:
        sys.exit("bench.py times single-layer, HBM-resident workloads (C0, C1, C4)")
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    torch.cuda.set_device(0)
    r = Rekv.for_workload(w)

    def dev(x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(tdt).to("cuda:0")

    # inputs: seeded, generated frame by frame on the host, resident in HBM before timing
    step = 64
    dq = torch.cat([dev(W.frames_q(w, f, min(f + step, w.n_frames))) for f in range(0, w.n_frames, step)])
    dk = torch.cat([dev(W.frames_k(w, f, min(f + step, w.n_frames))) for f in range(0, w.n_frames, step)])
    dv = torch.cat([dev(W.frames_v(w, f, min(f + step, w.n_frames))) for f in range(0, w.n_frames, step)])
    qs = [W.question_qkv(w, i) for i in range(w.n_questions)]
    q_q, q_k, q_v = (dev(np.stack([x[j] for x in qs])) for j in range(3))
    n_chunks = w.n_frames // w.chunk_frames
    d_prime = w.d_prime
    out = torch.empty_like(dq)
    fk = torch.empty((w.n_frames, d_prime), dtype=torch.float32, device="cuda:0")
    ret_shape = (w.n_questions, w.top_k * w.tokens_per_frame, w.n_kv_heads, w.head_dim)
    gk, gv = torch.empty(ret_shape, dtype=tdt, device="cuda:0"), torch.empty(ret_shape, dtype=tdt, device="cuda:0")
    qa_out = torch.empty_like(q_q)

    names = ["encode", "frame_keys", "retrieve", "gather", "qa"]
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] for _ in range(args.steps)]

    def one_step(ev=None):
        if ev: ev[0].record()
        r.encode_chunk(dq, dk, dv, 0, w.l_x, n_chunks, w.l_l, out=out)
        if ev: ev[1].record()
        r.frame_keys(dk, w.n_frames, out=fk)
        if ev: ev[2].record()
        idx, _, _ = r.retrieve_topk(fk, w.n_frames, q_q, w.top_k)
        if ev: ev[3].record()
        r.gather_kv(dk, dv, idx, dst_k=gk, dst_v=gv)
        if ev: ev[4].record()
        r.qa_attention(q_q, gk, gv, q_k, q_v, out=qa_out)
        if ev: ev[5].record()
        return idx

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        idx = one_step(evs[s])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms = {n: sum(e[i].elapsed_time(e[i + 1]) for e in evs) / args.steps for i, n in enumerate(names)}
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = w.n_tokens / (elapsed / args.steps)

    # the same stream encoded chunk by chunk (one launch per chunk, as a live stream arrives)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for c in range(n_chunks):
        r.encode_chunk(dq[c * w.l_x:(c + 1) * w.l_x], dk, dv, c * w.l_x, w.l_x, 1, w.l_l,
                       out=out[c * w.l_x:(c + 1) * w.l_x])
    torch.cuda.synchronize()
    streaming_s = time.perf_counter() - t1

    planted = [set(W.planted_frames(w, i).tolist()) <= set(idx[i].tolist()) for i in range(w.n_questions)]
    fl = encode_flops(w)
    if w.dtype == "bf16":
        bound, peak = "mfma", PEAK_BF16_TFLOPS
    else:
        bound, peak = "alu", PEAK_FP32_VALU_TFLOPS
    achieved = fl / (ms["encode"] * 1e-3) / 1e12
    es = 2 if w.dtype == "bf16" else 4
    gather_bytes = 2 * 2 * w.n_questions * w.top_k * w.tokens_per_frame * d_prime * es   # K and V, read + write
    fk_bytes = w.n_tokens * d_prime * es + w.n_frames * d_prime * 4
    result = {
        "metric": "video tokens/s encoded (windowed attn, MFMA %); retrieval+QA latency ms (HBM GB/s)",
        "value": tokens_per_s, "unit": "video tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_frames} frames x {w.tokens_per_frame} tokens, "
                               f"Hq/Hkv/D {w.n_q_heads}/{w.n_kv_heads}/{w.head_dim}, chunk {w.l_x} tokens, "
                               f"window {w.l_l} tokens, {w.n_questions} question(s) of {w.n_q_tokens} tokens, "
                               f"top-k {w.top_k}; one layer; a step = encode all {n_chunks} chunks in one "
                               f"launch + frame vectors + retrieval + gather + QA attention",
                   "n_chunks_per_launch": n_chunks},
        "roofline": {"bound": bound, "kernel": "attn_bf16_kernel (rekv_encode_chunk)" if w.dtype == "bf16"
                     else "attn_f32_kernel (rekv_encode_chunk)",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
                     "algorithmic_flop_per_launch": fl, "avg_launch_ms": ms["encode"]},
        "kernel_ms": ms,
        "retrieval_qa_latency_ms": ms["retrieve"] + ms["gather"] + ms["qa"],
        "encode_only_tokens_per_s": w.n_tokens / (ms["encode"] * 1e-3),
        "streaming_tokens_per_s": w.n_tokens / streaming_s,
        "hbm": {"gather_GBs": gather_bytes / (ms["gather"] * 1e-3) / 1e9,
                "frame_keys_GBs": fk_bytes / (ms["frame_keys"] * 1e-3) / 1e9,
                "qa_TFLOPs": qa_flops(w) / (ms["qa"] * 1e-3) / 1e12, "peak_GBs": PEAK_HBM_GBS},
        "planted_frames_retrieved": all(planted),
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
