"""Turns rocprofv3 CSV output of bench.py runs into the short text summaries kept under profiles/.

    python -m paper_2503_00540_amd.profile_summary trace   <dir> <out.txt> "<command>" [--bench-json FILE]
    python -m paper_2503_00540_amd.profile_summary traffic <fetch_dir> <write_dir> <out.txt> "<fetch cmd>" "<write cmd>"
    python -m paper_2503_00540_amd.profile_summary cycles  <dir> [<dir> ...] <out.txt> "<command>" [--zero-run <dir> "<command>"]

<dir> is a rocprofv3 output directory (-d) holding *_kernel_trace.csv and, for counter runs,
*_counter_collection.csv.  Kernels are grouped by name and grid size, because one kernel name
serves launches of very different shapes (all chunks of a stream in one launch, or one chunk).
Nothing here touches a GPU.
"""
from __future__ import annotations

import collections
import csv
import glob
import hashlib
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ENCODE_KERNEL_SOURCE = os.path.join(ROOT, "paper_2503_00540_amd", "csrc", "attention_bf16.hip")
ENCODE_FLOP_C1 = 2.2518e12          # algorithmic FLOP of one C1 encode launch (bench.encode_flops)
N_SIMD, N_XCD = 1024, 8


def _one(d, pattern):
    hits = sorted(glob.glob(os.path.join(d, "**", pattern), recursive=True))
    if len(hits) != 1:
        raise FileNotFoundError(f"expected one {pattern} under {d}, found {len(hits)}")
    return hits[0]


def short_name(name: str) -> str:
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    name = re.sub(r"^void ", "", name)
    m = re.match(r"(?:rekv::)?([\w:]+(?:<[^(]*>)?)\(", name)
    return m.group(1) if m else name[:60]


def _library_kernel(name: str) -> bool:
    return "rekv::" in name


def load_trace(d):
    rows = list(csv.DictReader(open(_one(d, "*kernel_trace.csv"))))
    out = {}
    for r in rows:
        grid = int(r.get("Grid_Size_X", r.get("Grid_Size", 0)) or 0) * max(int(r.get("Grid_Size_Y", 1) or 1), 1) * \
            max(int(r.get("Grid_Size_Z", 1) or 1), 1)
        out[r["Dispatch_Id"]] = (r["Kernel_Name"], int(r["End_Timestamp"]) - int(r["Start_Timestamp"]), grid)
    return out


def trace_table(d):
    groups = collections.defaultdict(list)
    for name, ns, grid in load_trace(d).values():
        if _library_kernel(name):
            groups[(short_name(name), grid)].append(ns)
    total = sum(sum(v) for v in groups.values())
    lines = ["%-58s %10s %6s %11s %11s %11s %7s" % ("kernel", "threads", "calls", "avg_us", "min_us", "max_us", "time%")]
    for (name, grid), v in sorted(groups.items(), key=lambda kv: -sum(kv[1])):
        lines.append("%-58s %10d %6d %11.1f %11.1f %11.1f %7.2f" % (name[:58], grid, len(v), sum(v) / len(v) / 1e3,
                                                                   min(v) / 1e3, max(v) / 1e3, 100.0 * sum(v) / total))
    return "\n".join(lines), groups


def load_counters(d):
    """{(kernel, grid): {counter: [values per dispatch]}} and the durations of the same dispatches."""
    trace = load_trace(d)
    per = collections.defaultdict(lambda: collections.defaultdict(dict))
    for r in csv.DictReader(open(_one(d, "*counter_collection.csv"))):
        name, ns, grid = trace[r["Dispatch_Id"]]
        if _library_kernel(name):
            key = (short_name(name), grid)
            per[key][r["Dispatch_Id"]][r["Counter_Name"]] = float(r["Counter_Value"])
            per[key][r["Dispatch_Id"]]["__ns"] = ns
    return per


def _largest(per, kernel_substr):
    """Counters of the longest dispatch among the kernels whose name holds kernel_substr."""
    best = None
    for (name, grid), disp in per.items():
        if kernel_substr in name:
            for vals in disp.values():
                if best is None or vals["__ns"] > best[1]["__ns"]:
                    best = ((name, grid), vals)
    return best


def cmd_trace(argv):
    d, out, command = argv[0], argv[1], argv[2]
    bench_json = argv[argv.index("--bench-json") + 1] if "--bench-json" in argv else None
    table, groups = trace_table(d)
    text = ["rocprofv3 kernel trace, library kernels only, grouped by kernel and total thread count.  MI355X, ROCm 7.2.", "",
            f"command: {command}", f"source : {os.path.basename(_one(d, '*kernel_trace.csv'))}", "", table, ""]
    b = None
    if bench_json:
        import json
        b = json.loads(open(bench_json).read().strip().splitlines()[-1])
    enc = [(k, v) for k, v in groups.items() if "attn_bf16_kernel<128, true" in k[0]]
    if enc:
        (name, grid), v = max(enc, key=lambda kv: kv[0][1])
        avg = sum(v) / len(v)
        text.append(f"Encode launch of the timed step: {name} with {grid} threads, {len(v)} calls, average {avg / 1e3:.1f} us "
                    f"(rows of the same kernel with fewer threads: the one-chunk-per-launch streaming calls, and for the "
                    f"offloaded-KV workload the stream's first, shorter segment).")
        if "--no-extras" not in command:
            text.append("This run includes the benchmark's extras: the launches on all-zero inputs are among those calls and "
                        "pull the average down (they are the fastest ones); the trace of the --no-extras command holds the "
                        "timed configuration alone.")
        # the workload's own algorithmic FLOP per launch, as the benchmark line of the same run states it
        flop = b["roofline"]["algorithmic_flop_per_launch"] if b else ENCODE_FLOP_C1
        what = b["config"]["workload"].split(":")[0] if b else "C1-7B-1layer"
        text.append(f"{what}: {flop:.4e} algorithmic FLOP per launch -> {flop / avg / 1e3:.0f} TFLOP/s = "
                    f"{100 * flop / avg / 1e3 / 2500:.1f} % of the 2.5 PFLOP/s bf16 MFMA peak.")
    if b and "offloaded" in b["config"]["workload"] and enc:
        text.append(f"Under the profiler the offload copies on the side stream slow the encode launches they overlap: the "
                    f"step's first launch, which overlaps none, is the minimum ({min(v) / 1e3:.1f} us); without the profiler "
                    f"all launches of this workload take about that long (benchmark line of a plain run: roofline.frac 0.41-0.43).")
    if b:
        text.append(f"bench.py's own HIP-event average of the encode launch in the same run: {b['roofline']['avg_launch_ms'] * 1e3:.1f} us; "
                    f"roofline.frac {b['roofline']['frac']:.3f}.")
    open(out, "w").write("\n".join(text) + "\n")


def cmd_traffic(argv):
    fetch_dir, write_dir, out, fetch_cmd, write_cmd = argv[:5]
    pf, pw = load_counters(fetch_dir), load_counters(write_dir)
    text = ["HBM traffic per dispatch from two rocprofv3 counter runs of the benchmark (FETCH_SIZE, then WRITE_SIZE; KiB).", "",
            f"commands: {fetch_cmd}", f"          {write_cmd}", "source  : *_counter_collection.csv, longest dispatch of each (kernel, thread count)", "",
            "%-58s %10s %14s %14s" % ("kernel", "threads", "FETCH_SIZE", "WRITE_SIZE")]
    for key in pf:
        fe = max(v.get("FETCH_SIZE", 0.0) for v in pf[key].values())
        wr = max((v.get("WRITE_SIZE", 0.0) for v in pw.get(key, {}).values()), default=float("nan"))
        text.append("%-58s %10d %14.1f %14.1f" % (key[0][:58], key[1], fe, wr))
    copy_f, copy_w = _largest(pf, "probe_copy_kernel"), _largest(pw, "probe_copy_kernel")
    enc_f, enc_w = _largest(pf, "attn_bf16_kernel<128, true"), _largest(pw, "attn_bf16_kernel<128, true")
    if copy_f and copy_w and enc_f and enc_w:
        kib = 1 << 20                                     # the probe copies 1 GiB each way
        ff, fw = kib / copy_f[1]["FETCH_SIZE"], kib / copy_w[1]["WRITE_SIZE"]
        rd, wr = enc_f[1]["FETCH_SIZE"] * ff * 1024, enc_w[1]["WRITE_SIZE"] * fw * 1024
        text += ["", "Calibration on the copy kernel of the same runs (rekv_probe_copy moves 1 GiB = 1,048,576 KiB each way):",
                 f"  FETCH_SIZE reads {copy_f[1]['FETCH_SIZE']:.0f} -> factor {ff:.3f};  WRITE_SIZE reads {copy_w[1]['WRITE_SIZE']:.0f} -> factor {fw:.3f}",
                 f"Encode launch ({enc_f[0][0]}, {enc_f[0][1]} threads): read {rd / 1e6:.0f} MB, written {wr / 1e6:.0f} MB, total {(rd + wr) / 1e6:.0f} MB.",
                 "Algorithmic bytes of the C1 launch: Q 359.7 MB + K 51.4 MB + V 51.4 MB read, O 359.7 MB written = 822 MB.", "",
                 f"traffic_bytes_per_launch: {int(rd + wr)}",
                 f"kernel_source_sha256: {hashlib.sha256(open(ENCODE_KERNEL_SOURCE, 'rb').read()).hexdigest()}"]
    open(out, "w").write("\n".join(text) + "\n")


def _zero_input_block(d, command):
    """Clock and MFMA-busy share of the encode launch on all-zero inputs: in a run of the default command
    (extras on) the whole-stream encode kernel is launched on the benchmark's inputs and, for the zero-input
    diagnostic, on zeros; the zero-input launches are the shortest dispatches of that (kernel, thread count)."""
    per = load_counters(d)
    enc = [(key, disp) for key, disp in per.items() if "attn_bf16_kernel<128, true" in key[0]]
    if not enc:
        return []
    (name, grid), disp = max(enc, key=lambda kv: kv[0][1])
    vals = sorted(disp.values(), key=lambda v: v["__ns"])
    lines = ["== encode launch on all-zero inputs against the same launch on the benchmark's inputs",
             f"  command: {command}",
             f"  {name}, {grid} threads, {len(vals)} dispatches; shortest = zero inputs, longest = benchmark inputs"]
    for label, v in (("zero inputs", vals[0]), ("benchmark inputs", vals[-1])):
        cyc = v["GRBM_GUI_ACTIVE"] / N_XCD
        lines.append(f"  {label:17s}: {v['__ns'] / 1e3:8.1f} us, {cyc:.4g} clocks -> {cyc / v['__ns']:.2f} GHz; MFMA pipes busy "
                     f"{100 * v['SQ_VALU_MFMA_BUSY_CYCLES'] / N_SIMD / cyc:.1f} %; SQ_INSTS_MFMA {v['SQ_INSTS_MFMA']:.6g}")
    lines.append("  Same instruction stream and about the same number of clocks; the clock the chip grants differs.")
    lines.append("")
    return lines


def cmd_cycles(argv):
    zero_dir = zero_cmd = None
    if "--zero-run" in argv:
        i = argv.index("--zero-run")
        zero_dir, zero_cmd = argv[i + 1], argv[i + 2]
        argv = argv[:i] + argv[i + 3:]
    dirs, out, command = argv[:-2], argv[-2], argv[-1]
    text = ["Cycle budget of the encode launch (all chunks of the C1 stream) and of the register-resident MFMA probe, from rocprofv3",
            "counter runs of the benchmark.  SQ_*_CYCLES and SQ_ACTIVE_* / SQ_WAIT_* count in units of 4 clocks, summed over the chip;",
            "SQ_VALU_MFMA_BUSY_CYCLES counts clocks summed over the 1024 SIMDs; GRBM_GUI_ACTIVE counts clocks summed over the 8 XCDs.", "",
            f"command (one run per counter set): {command}", ""]
    for sub, label in (("attn_bf16_kernel<128, true", "encode launch"), ("probe_mfma_kernel", "MFMA probe (independent 32x32x16 bf16 MFMAs on N(0,1)-like operands)")):
        merged = {}
        for d in dirs:
            best = _largest(load_counters(d), sub)
            if best:
                for k, v in best[1].items():
                    merged.setdefault(k if k != "__ns" else f"duration_ns[{os.path.basename(d.rstrip('/'))}]", v)
        if not merged:
            continue
        text.append(f"== {label}")
        for k in sorted(merged):
            text.append("  %-44s %.6g" % (k, merged[k]))
        durs = [v for k, v in merged.items() if k.startswith("duration_ns")]
        if "GRBM_GUI_ACTIVE" in merged:
            gui_dir = [k for k in merged if k.startswith("duration_ns")]
            # the run that collected GRBM_GUI_ACTIVE: pair it with that run's duration
            for d in dirs:
                best = _largest(load_counters(d), sub)
                if best and "GRBM_GUI_ACTIVE" in best[1]:
                    ns = best[1]["__ns"]
                    cyc = best[1]["GRBM_GUI_ACTIVE"] / N_XCD
                    text.append(f"  clock during the launch = GRBM_GUI_ACTIVE / {N_XCD} / duration = {cyc / ns:.2f} GHz (2.5 PFLOP/s assumes 2.4 GHz)")
                    if "SQ_VALU_MFMA_BUSY_CYCLES" in best[1]:
                        text.append(f"  MFMA pipes busy = SQ_VALU_MFMA_BUSY_CYCLES / ({N_SIMD} SIMDs x {cyc:.4g} clocks) = "
                                    f"{100 * best[1]['SQ_VALU_MFMA_BUSY_CYCLES'] / N_SIMD / cyc:.1f} %")
        if "SQ_WAVE_CYCLES" in merged:
            wc = merged["SQ_WAVE_CYCLES"]
            for k in ("SQ_WAIT_INST_ANY", "SQ_WAIT_ANY", "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_VALU", "SQ_ACTIVE_INST_LDS"):
                if k in merged:
                    text.append(f"  {k} / SQ_WAVE_CYCLES = {100 * merged[k] / wc:.1f} % of resident wave time")
        if "SQ_INSTS_VALU" in merged and "SQ_INSTS_MFMA" in merged:
            text.append(f"  vector instructions per MFMA (SQ_INSTS_VALU / SQ_INSTS_MFMA, MFMAs included) = {merged['SQ_INSTS_VALU'] / merged['SQ_INSTS_MFMA']:.2f}")
        text.append("")
    if zero_dir:
        text += _zero_input_block(zero_dir, zero_cmd)
    open(out, "w").write("\n".join(text) + "\n")


def main(argv=None):
    argv = sys.argv[1:] if argv is None else argv
    if not argv or argv[0] not in ("trace", "traffic", "cycles"):
        sys.exit(__doc__)
    {"trace": cmd_trace, "traffic": cmd_traffic, "cycles": cmd_cycles}[argv[0]](argv[1:])


if __name__ == "__main__":
    main()
