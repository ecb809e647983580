"""Host-side measurement helpers: the summariser that turns rocprofv3 CSVs into the text files under
profiles/, and the benchmark's lookup of the measured HBM traffic.  No GPU, no rocprofv3: the CSVs
are written here with the columns the profiler emits."""
import csv
import hashlib
import os
import re

import bench
from paper_2503_00540_amd import profile_summary as PS

ENC = "void rekv::(anonymous namespace)::attn_bf16_kernel<128, true, false, false>(rekv::(anonymous namespace)::KernelArgs)"
COPY = "rekv::(anonymous namespace)::probe_copy_kernel(uint4*, uint4 const*, long)"


def _write_run(d, dispatches, counters=None):
    """dispatches: [(id, kernel, grid_x, start_ns, end_ns)]; counters: {id: {name: value}}."""
    os.makedirs(d)
    with open(os.path.join(d, "p_kernel_trace.csv"), "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Dispatch_Id", "Kernel_Name", "Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z", "Start_Timestamp", "End_Timestamp"])
        for i, name, grid, t0, t1 in dispatches:
            w.writerow([i, name, grid, 1, 1, t0, t1])
    if counters is not None:
        with open(os.path.join(d, "p_counter_collection.csv"), "w", newline="") as f:
            w = csv.writer(f)
            w.writerow(["Dispatch_Id", "Counter_Name", "Counter_Value"])
            for i, vals in counters.items():
                for k, v in vals.items():
                    w.writerow([i, k, v])


def test_trace_summary_groups_by_kernel_and_grid(tmp_path):
    d = str(tmp_path / "run")
    _write_run(d, [(1, ENC, 2883584, 0, 2_000_000), (2, ENC, 2883584, 3_000_000, 5_200_000),
                   (3, ENC, 123904, 6_000_000, 6_020_000), (4, "void at::native::fill(float*)", 64, 7_000_000, 7_001_000)])
    out = str(tmp_path / "trace.txt")
    PS.main(["trace", d, out, "rocprofv3 ... -- python3 bench.py --no-cpu-baseline --no-extras"])
    text = open(out).read()
    rows = [l for l in text.splitlines() if l.startswith("attn_bf16_kernel")]
    assert len(rows) == 2 and "at::native" not in text                 # two shapes of one kernel; foreign kernels left out
    big = [l for l in rows if " 2883584 " in l][0].split()
    assert big[-6:-1] == ["2883584", "2", "2100.0", "2000.0", "2200.0"]
    m = re.search(r"average ([\d.]+) us", text)
    assert float(m.group(1)) == 2100.0
    assert "command: rocprofv3 ... -- python3 bench.py" in text


def test_traffic_summary_calibrates_on_the_copy_kernel(tmp_path):
    gib_kib = 1 << 20
    fetch, write = str(tmp_path / "fetch"), str(tmp_path / "write")
    disp = [(1, COPY, 2097152, 0, 360_000), (2, ENC, 2883584, 400_000, 2_600_000)]
    _write_run(fetch, disp, {1: {"FETCH_SIZE": gib_kib / 2}, 2: {"FETCH_SIZE": 250_000.0}})      # the counter reads half
    _write_run(write, disp, {1: {"WRITE_SIZE": float(gib_kib)}, 2: {"WRITE_SIZE": 300_000.0}})
    out = str(tmp_path / "traffic.txt")
    PS.main(["traffic", fetch, write, out, "fetch command", "write command"])
    text = open(out).read()
    m = re.search(r"^traffic_bytes_per_launch: (\d+)$", text, re.M)
    assert m and int(m.group(1)) == int((250_000.0 * 2.0 + 300_000.0 * 1.0) * 1024)
    h = re.search(r"^kernel_source_sha256: ([0-9a-f]{64})$", text, re.M)
    src = os.path.join(bench.ROOT, bench.ENCODE_KERNEL_SOURCE)
    assert h and h.group(1) == hashlib.sha256(open(src, "rb").read()).hexdigest()


def test_cycle_summary_reports_clock_and_busy_share(tmp_path):
    d = str(tmp_path / "cyc")
    ns = 2_000_000
    clocks = 1.6 * ns                                            # 1.6 GHz
    _write_run(d, [(1, ENC, 2883584, 0, ns)],
               {1: {"GRBM_GUI_ACTIVE": clocks * PS.N_XCD, "SQ_VALU_MFMA_BUSY_CYCLES": 0.5 * clocks * PS.N_SIMD, "SQ_INSTS_MFMA": 7e7}})
    out = str(tmp_path / "cycles.txt")
    PS.main(["cycles", d, out, "counter command"])
    text = open(out).read()
    assert "= 1.60 GHz" in text and "= 50.0 %" in text


def test_bench_quotes_traffic_only_for_the_source_it_was_measured_on(tmp_path, monkeypatch):
    value, source = bench.measured_traffic("C1-7B-1layer")
    assert (value is None) or (value > 0 and "profiles/" in source)
    assert bench.measured_traffic("C3-28layers")[0] is None      # no counter summary for that workload
    # a summary measured on another version of the kernel source is not quoted
    root = tmp_path / "tree"
    (root / "profiles").mkdir(parents=True)
    (root / "paper_2503_00540_amd" / "csrc").mkdir(parents=True)
    (root / bench.ENCODE_KERNEL_SOURCE).write_text("// kernel v2\n")
    sha_old = hashlib.sha256(b"// kernel v1\n").hexdigest()
    (root / bench.TRAFFIC_PROFILE["C1-7B-1layer"]).write_text(f"traffic_bytes_per_launch: 123\nkernel_source_sha256: {sha_old}\n")
    monkeypatch.setattr(bench, "ROOT", str(root))
    value, why = bench.measured_traffic("C1-7B-1layer")
    assert value is None and "another version" in why
    sha_new = hashlib.sha256(b"// kernel v2\n").hexdigest()
    (root / bench.TRAFFIC_PROFILE["C1-7B-1layer"]).write_text(f"traffic_bytes_per_launch: 123\nkernel_source_sha256: {sha_new}\n")
    assert bench.measured_traffic("C1-7B-1layer")[0] == 123
