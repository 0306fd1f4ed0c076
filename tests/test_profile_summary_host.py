"""Host logic of paper_2409_07146_amd.profile_summary on small hand-written CSV files in rocprofv3's column
layout: kernel names are shortened, the two apply launches are told apart by grid size, the traffic counters
are scaled by what they read for the copy probe (whose true bytes are known), and the JSON that bench.py
puts into `roofline.traffic` carries bytes per launch."""
import csv
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

INTRA = "_ZN3gsa18chunk_intra_kernelIDF16bLi64ELb0ELb0EEEvNS_8ChunkMapEiiifNS_9IntraArgsIT_EE"
APPLY = "_ZN3gsa12apply_kernelIDF16bLi64ELb0ELb0EEEvNS_8ChunkMapEiNS_9ApplyArgsIT_EE"
SCANR = "_ZN3gsa11scan_kernelIDF16bLi64ELi64ELb1ELi0EEEvNS_8ChunkMapEiiiiNS_8ScanArgsIT_EE"
COPY = "_ZN3gsa17copy_probe_kernelEPvPKvm"


def _write(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(header)
        w.writerows(rows)


def _counter_rows(counter, values):
    hdr = ["Correlation_Id", "Dispatch_Id", "Agent_Id", "Queue_Id", "Process_Id", "Thread_Id", "Grid_Size", "Kernel_Id",
           "Kernel_Name", "Workgroup_Size", "LDS_Block_Size", "Scratch_Size", "VGPR_Count", "Accum_VGPR_Count",
           "SGPR_Count", "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"]
    rows = []
    for i, (name, grid, val) in enumerate(values):
        rows.append([i, i, "Agent 1", 1, 1, 1, grid, 1, name, 256, 0, 0, 64, 0, 96, counter, float(val), 1000 * i, 1000 * i + 500])
    return hdr, rows


def test_summaries_from_small_csv_files(tmp_path):
    kt = tmp_path / "kt" / "bench_kernel_trace.csv"
    hdr = ["Kind", "Agent_Id", "Queue_Id", "Stream_Id", "Thread_Id", "Dispatch_Id", "Kernel_Id", "Kernel_Name",
           "Correlation_Id", "Start_Timestamp", "End_Timestamp", "LDS_Block_Size", "Scratch_Size", "VGPR_Count",
           "Accum_VGPR_Count", "SGPR_Count", "Workgroup_Size_X", "Workgroup_Size_Y", "Workgroup_Size_Z", "Grid_Size_X",
           "Grid_Size_Y", "Grid_Size_Z"]
    def row(i, name, t0, t1, gx, gy=1, gz=1):
        return ["KERNEL_DISPATCH", "Agent 1", 1, 1, 1, i, 1, name, i, t0, t1, 0, 0, 64, 0, 96, 256, 1, 1, gx, gy, gz]
    _write(str(kt), hdr, [row(0, INTRA, 0, 130000, 65536, 4), row(1, INTRA, 200000, 328000, 65536, 4),
                          row(2, APPLY, 400000, 440000, 1024, 256, 4), row(3, APPLY, 500000, 600000, 1024, 256, 12),
                          row(4, SCANR, 700000, 760000, 131072)])
    # the copy probe moves 256 MiB each way; FETCH_SIZE reads half of that in KiB, WRITE_SIZE all of it
    mib = 1 << 20
    h, r = _counter_rows("FETCH_SIZE", [(COPY, 1, 256 * mib / 1024 / 2), (INTRA, 262144, 100000.0), (INTRA, 262144, 120000.0)])
    _write(str(tmp_path / "f" / "pmc_counter_collection.csv"), h, r)
    h, r = _counter_rows("WRITE_SIZE", [(COPY, 1, 256 * mib / 1024), (INTRA, 262144, 50000.0), (INTRA, 262144, 50000.0)])
    _write(str(tmp_path / "w" / "pmc_counter_collection.csv"), h, r)
    out = tmp_path / "out"
    os.makedirs(out)
    cmd = [sys.executable, "-m", "paper_2409_07146_amd.profile_summary", "--kernel-trace", str(tmp_path / "kt"),
           "--fetch", str(tmp_path / "f"), "--write", str(tmp_path / "w"), "--out", str(out), "--workload", "toy"]
    subprocess.run(cmd, cwd=ROOT, check=True)
    trace = open(out / "toy_fwd_bwd_kernel_trace.txt").read()
    assert "chunk_intra_kernel<bf16,64>" in trace and "scan_kernel<bf16,64,reverse>" in trace
    assert "apply_kernel<bf16,64> forward (o)" in trace and "apply_kernel<bf16,64> backward (dq,dk,dv)" in trace
    line = [l for l in trace.splitlines() if l.startswith("chunk_intra_kernel")][0].split()
    assert int(line[1]) == 2 and abs(float(line[3]) - 129.0) < 1e-6      # two calls, 130 and 128 us
    rec = json.load(open(out / "hbm_traffic_toy.json"))["kernels"]["chunk_intra_kernel"]
    # fetched: mean 110000 KiB x 2.0 (the probe's factor); written: 50000 KiB x 1.0
    assert abs(rec["fetch_bytes"] - 110000 * 1024 * 2.0) < 1.0
    assert abs(rec["write_bytes"] - 50000 * 1024 * 1.0) < 1.0
