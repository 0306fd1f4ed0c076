"""Turns raw rocprofv3 output of `bench.py` into the short text summaries kept under profiles/.

It computes nothing of the operator: it reads the CSV files rocprofv3 writes (kernel trace, counter
collection) and prints per-kernel averages.  Four profiler runs of the same bench command feed it, each in
a directory of its own (counters are collected one group per run):

    cd /tmp && export TMPDIR=/tmp        # R = repository root, OUT = a scratch directory for the raw output
    rocprofv3 --kernel-trace --output-format csv -d $OUT/kt -o bench -- python3 $R/bench.py --steps 20 --warmup 5 --no-cpu-baseline
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d $OUT/pmc_f -o pmc -- python3 $R/bench.py --steps 3 --warmup 1 --decode-steps 16 --no-cpu-baseline
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d $OUT/pmc_w -o pmc -- python3 $R/bench.py --steps 3 --warmup 1 --decode-steps 16 --no-cpu-baseline
    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_MFMA GRBM_GUI_ACTIVE --output-format csv -d $OUT/pmc_sq -o pmc -- python3 $R/bench.py --steps 3 --warmup 1 --decode-steps 16 --no-cpu-baseline
    python3 -m paper_2409_07146_amd.profile_summary --kernel-trace $OUT/kt --fetch $OUT/pmc_f --write $OUT/pmc_w --sq $OUT/pmc_sq --out profiles --workload layer_1p3b

A fifth run, summarised with --insts, gives the executed instruction mix and the LDS bank conflicts:

    rocprofv3 --pmc SQ_WAVES SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_INSTS_VMEM SQ_INSTS_VALU_TRANS_F32 SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE --output-format csv -d $OUT/pmc_in -o pmc -- python3 $R/bench.py --steps 3 --warmup 1 --decode-steps 16 --no-cpu-baseline

Outputs: <workload>_fwd_bwd_kernel_trace.txt, <workload>_fwd_bwd_hbm_traffic.txt, <workload>_mfma_utilisation.txt,
<workload>_instruction_mix.txt and hbm_traffic_<workload>.json (bytes per launch and kernel, which bench.py puts into `roofline.traffic`).
"""
import argparse
import collections
import csv
import glob
import json
import os
import re

MFMA_BF16_PEAK = 2.5e15      # MI355X dense bf16, FLOP/s
SIMDS = 256 * 4              # compute units x SIMDs


def short(name):
    """A readable kernel name from the mangled one."""
    n = re.sub(r"^_ZN3gsa\d+", "", name)
    m = re.match(r"(scan_kernel)I(DF16b|f)Li(\d+)ELi\d+ELb([01])ELi(\d)", n)
    if m:
        mode = {"0": "", "1": " summary pass", "2": " segments"}[m.group(5)]
        return "scan_kernel<%s,%s,%s>%s" % ("bf16" if m.group(2) == "DF16b" else "f32", m.group(3),
                                            "reverse" if m.group(4) == "1" else "forward", mode)
    m = re.match(r"decode_kernelI(DF16b|f)Li(\d+)ELi\d+ELb[01]ELi(\d+)ELi(\d+)E", n)
    if m:
        return "decode_kernel<%s,%s> %s waves, %s" % ("bf16" if m.group(1) == "DF16b" else "f32", m.group(2), m.group(3),
                                                     "whole pair" if m.group(4) == "0" else m.group(4) + " pieces per pair")
    m = re.match(r"([a-z_]+_kernel)I(DF16b|f)Li(\d+)(?:ELb([01])ELb([01]))?", n)
    if m:
        base = "%s<%s,%s>" % (m.group(1), "bf16" if m.group(2) == "DF16b" else "f32", m.group(3))
        if m.group(4) is not None:   # the two template switches after the slot count
            if m.group(1) == "apply_kernel":
                base += (" feature map" if m.group(4) == "1" else "") + (" epilogue" if m.group(5) == "1" else "")
            else:
                base += (" general form" if m.group(4) == "1" else "") + (" feature map" if m.group(5) == "1" else "")
        return base
    if "copy_probe_kernel" in n:
        return "copy_probe_kernel"
    return n[:48]


def find_csv(directory, suffix):
    hits = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit("no *%s under %s" % (suffix, directory))
    return hits[0]


def split_apply(rows):
    """The apply kernel is launched twice per step; its launches are told apart by grid size."""
    def grid(r):   # the counter file has one column, the kernel trace one per dimension
        if "Grid_Size" in r:
            return int(r["Grid_Size"])
        return int(r["Grid_Size_X"]) * int(r["Grid_Size_Y"]) * int(r["Grid_Size_Z"])
    grids = sorted({grid(r) for r in rows if "apply_kernel" in r["Kernel_Name"]})

    def name(r):
        s = short(r["Kernel_Name"])
        if s.startswith("apply_kernel") and len(grids) == 2:
            s += " forward (o)" if grid(r) == grids[0] else " backward (dq,dk,dv)"
        return s
    return name


def kernel_trace(directory):
    rows = list(csv.DictReader(open(find_csv(directory, "kernel_trace.csv"))))
    name = split_apply(rows)
    dur = collections.defaultdict(list)
    for r in rows:
        dur[name(r)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) * 1e-3)   # us
    return dur


def counters(directory):
    rows = list(csv.DictReader(open(find_csv(directory, "counter_collection.csv"))))
    name = split_apply(rows)
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    dur = collections.defaultdict(list)
    for r in rows:
        agg[name(r)][r["Counter_Name"]].append(float(r["Counter_Value"]))
        dur[name(r)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) * 1e-3)
    mean = {k: {c: sum(v) / len(v) for c, v in d.items()} for k, d in agg.items()}
    calls = {k: max(len(v) for v in d.values()) for k, d in agg.items()}
    return mean, calls, {k: sum(v) / len(v) for k, v in dur.items()}


SLOT = {"chunk_intra_kernel": "chunk_intra_kernel", "chunk_fwd_kernel": "chunk_fwd_kernel", "chunk_dz_kernel": "chunk_dz_kernel",
        "gate_kernel": "gate_kernel", "copy_probe_kernel": "copy_probe_kernel", "decode_kernel": "decode_kernel"}


def slot_of(name):
    """The name bench.py's per-kernel timing uses for this kernel."""
    if name.startswith("scan_kernel"):
        return "scan_bwd_kernel" if "reverse" in name else "scan_fwd_kernel"
    if name.startswith("apply_kernel"):
        return "apply_bwd_kernel" if "backward" in name else "apply_fwd_kernel"
    for k, v in SLOT.items():
        if name.startswith(k):
            return v
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--kernel-trace")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--sq")
    ap.add_argument("--insts", help="directory of the instruction-mix run (SQ_WAVES, SQ_INSTS_*, SQ_LDS_*)")
    ap.add_argument("--out", default="profiles")
    ap.add_argument("--workload", default="layer_1p3b")
    ap.add_argument("--command", default="python3 $R/bench.py", help="the profiled command, for the file headers")
    ap.add_argument("--trace-args", default="--steps 20 --warmup 5 --no-cpu-baseline",
                    help="the arguments the kernel-trace run gave the command, for the file header")
    ap.add_argument("--trace-name", default=None, help="file name of the kernel-trace summary (default <workload>_fwd_bwd_kernel_trace.txt)")
    ap.add_argument("--trace-note", default=None, help="replaces the paragraph on what a forward + backward step launches")
    args = ap.parse_args()
    os.makedirs(args.out, exist_ok=True)
    wl = args.workload

    if args.kernel_trace:
        dur = kernel_trace(args.kernel_trace)
        total = sum(sum(v) for v in dur.values())
        note = args.trace_note or (
            "Per step the forward launches gate, scan(forward), chunk_fwd, apply; the backward launches gate,\n"
            "scan(forward), chunk_dz, scan(reverse), chunk_intra, apply (dq, dk, dv in one launch).  scan(forward)\n"
            "therefore appears twice per step; its average mixes the forward's and the backward's launch.  The run\n"
            "also times the steps without recomputation, the decode steps and the 256 MiB copy probe.")
        with open(os.path.join(args.out, args.trace_name or "%s_fwd_bwd_kernel_trace.txt" % wl), "w") as f:
            f.write("rocprofv3 kernel trace of bench.py, workload %s.  Durations are End - Start of each dispatch.\n\n"
                    "command (run from /tmp with TMPDIR=/tmp; R = repository root, OUT = a scratch directory):\n"
                    "  rocprofv3 --kernel-trace --output-format csv -d $OUT/kt -o bench -- %s %s\n"
                    "summary: python3 -m paper_2409_07146_amd.profile_summary --kernel-trace $OUT/kt ...\n\n%s\n\n"
                    % (wl, args.command, args.trace_args, note))
            f.write("%-46s %7s %12s %10s %10s %7s\n" % ("kernel", "calls", "total_us", "avg_us", "median_us", "pct"))
            for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
                vs = sorted(v)
                f.write("%-46s %7d %12.1f %10.2f %10.2f %7.2f\n" % (k, len(v), sum(v), sum(v) / len(v), vs[len(vs) // 2],
                                                                 100.0 * sum(v) / total))

    if args.fetch and args.write:
        fe, nf, _ = counters(args.fetch)
        wr, _, _ = counters(args.write)
        probe_kib = 256 * 1024
        ff = probe_kib / fe["copy_probe_kernel"]["FETCH_SIZE"]
        fw = probe_kib / wr["copy_probe_kernel"]["WRITE_SIZE"]
        kern = {}
        with open(os.path.join(args.out, "%s_fwd_bwd_hbm_traffic.txt" % wl), "w") as f:
            f.write("HBM traffic per kernel launch from hardware counters, bench.py workload %s.\n\n"
                    "commands (run from /tmp with TMPDIR=/tmp; R = repository root, OUT = a scratch directory), one counter per run:\n"
                    "  rocprofv3 --pmc FETCH_SIZE --output-format csv -d $OUT/pmc_f -o pmc -- %s --steps 3 --warmup 1 --decode-steps 16 --no-cpu-baseline\n"
                    "  rocprofv3 --pmc WRITE_SIZE --output-format csv -d $OUT/pmc_w -o pmc -- %s --steps 3 --warmup 1 --decode-steps 16 --no-cpu-baseline\n"
                    "summary: python3 -m paper_2409_07146_amd.profile_summary --fetch $OUT/pmc_f --write $OUT/pmc_w ...\n\n"
                    "Calibration: copy_probe_kernel reads 256 MiB and writes 256 MiB per launch.  The counters (KiB per dispatch) read\n"
                    "FETCH_SIZE = %.0f and WRITE_SIZE = %.0f for it, so fetched bytes = FETCH_SIZE x %.3f KiB and written bytes =\n"
                    "WRITE_SIZE x %.3f KiB.  Averages are over all dispatches of a kernel in the run.\n\n"
                    % (wl, args.command, args.command, fe["copy_probe_kernel"]["FETCH_SIZE"], wr["copy_probe_kernel"]["WRITE_SIZE"], ff, fw))
            f.write("%-46s %6s %12s %12s %12s\n" % ("kernel", "calls", "fetched MB", "written MB", "total MB"))
            for k in fe:
                if k not in wr or "FETCH_SIZE" not in fe[k] or "WRITE_SIZE" not in wr[k]:
                    continue
                fb, wb = fe[k]["FETCH_SIZE"] * ff * 1024, wr[k]["WRITE_SIZE"] * fw * 1024
                kern[k] = {"fetch_bytes": round(fb), "write_bytes": round(wb)}
                f.write("%-46s %6d %12.1f %12.1f %12.1f\n" % (k, nf[k], fb / 1e6, wb / 1e6, (fb + wb) / 1e6))
        rec = {"workload": wl, "unit": "bytes per launch", "source": "%s_fwd_bwd_hbm_traffic.txt" % wl,
               "fetch_scale": ff, "write_scale": fw,
               "kernels": {slot_of(k): v for k, v in kern.items() if slot_of(k)}}
        with open(os.path.join(args.out, "hbm_traffic_%s.json" % wl), "w") as f:
            json.dump(rec, f, indent=1)

    if args.sq:
        sq, n, dur = counters(args.sq)
        with open(os.path.join(args.out, "%s_mfma_utilisation.txt" % wl), "w") as f:
            f.write("Matrix-core counters per kernel launch, bench.py workload %s.\n\n"
                    "command (run from /tmp with TMPDIR=/tmp; R = repository root, OUT = a scratch directory):\n"
                    "  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_MFMA GRBM_GUI_ACTIVE --output-format csv -d $OUT/pmc_sq -o pmc -- %s --steps 3 --warmup 1 --decode-steps 16 --no-cpu-baseline\n"
                    "summary: python3 -m paper_2409_07146_amd.profile_summary --sq $OUT/pmc_sq ...\n\n"
                    "mfma_busy %% = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE x %d SIMDs): the share of SIMD cycles with a matrix\n"
                    "instruction in flight (rocprofv3's MfmaUtil).  bf16 TFLOP/s = SQ_INSTS_VALU_MFMA_MOPS_BF16 x 512 / duration of the\n"
                    "dispatch under the profiler (counter collection slows a dispatch down; the kernel trace has the true durations),\n"
                    "%% of peak against %.1f PFLOP/s dense bf16.  Averages over all dispatches of a kernel in the run.\n"
                    "The busy-cycle counter reads about an eighth of what the operation counter implies (one instruction of 16x16x32\n"
                    "bf16 keeps a SIMD's matrix core busy for 8 passes of 4 cycles): on this chip it appears to be collected on one of\n"
                    "the 8 XCDs while the instruction and operation counters cover all of them, so mfma_busy %% x 8 is the figure that\n"
                    "agrees with the TFLOP/s column.\n\n"
                    % (wl, args.command, SIMDS, MFMA_BF16_PEAK / 1e15))
            f.write("%-46s %6s %12s %14s %12s %12s %10s\n" % ("kernel", "calls", "mfma_busy %", "MFMA instr", "bf16 GFLOP", "TFLOP/s",
                                                            "% of peak"))
            for k, d in sq.items():
                if "GRBM_GUI_ACTIVE" not in d or not d.get("GRBM_GUI_ACTIVE"):
                    continue
                busy = 100.0 * d.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) / (d["GRBM_GUI_ACTIVE"] * SIMDS)
                flop = d.get("SQ_INSTS_VALU_MFMA_MOPS_BF16", 0.0) * 512
                tf = flop / (dur[k] * 1e-6) / 1e12
                f.write("%-46s %6d %12.2f %14.0f %12.2f %12.1f %10.2f\n" % (k, n[k], busy, d.get("SQ_INSTS_MFMA", 0.0), flop / 1e9, tf,
                                                                          100.0 * tf * 1e12 / MFMA_BF16_PEAK))

    if args.insts:
        ins, n, _ = counters(args.insts)
        with open(os.path.join(args.out, "%s_instruction_mix.txt" % wl), "w") as f:
            f.write("Executed instructions per wave and LDS bank conflicts per kernel launch, bench.py workload %s.\n\n"
                    "command (run from /tmp with TMPDIR=/tmp; R = repository root, OUT = a scratch directory):\n"
                    "  rocprofv3 --pmc SQ_WAVES SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_INSTS_VMEM SQ_INSTS_VALU_TRANS_F32 SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE --output-format csv -d $OUT/pmc_in -o pmc -- %s --steps 3 --warmup 1 --decode-steps 16 --no-cpu-baseline\n"
                    "summary: python3 -m paper_2409_07146_amd.profile_summary --insts $OUT/pmc_in ...\n\n"
                    "Per wave = SQ_INSTS_* / SQ_WAVES (vector-ALU counts include the matrix instructions; trans = exp, log,\n"
                    "reciprocal and the like).  issue_us = vector-ALU instructions x 4 cycles x waves / (%d SIMDs x 2.4 GHz): the time\n"
                    "the launch's vector instructions take to issue if spread evenly, a floor that no occupancy shortens.\n"
                    "lds_conflict %% = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE: the share of LDS cycles lost to bank conflicts.\n"
                    "Averages over all dispatches of a kernel in the run.\n\n" % (wl, args.command, SIMDS))
            f.write("%-46s %6s %8s %8s %7s %7s %7s %7s %9s %14s\n" % ("kernel", "calls", "waves", "valu", "trans", "salu", "lds", "vmem",
                                                                   "issue_us", "lds_conflict %"))
            for k, d in ins.items():
                w = d.get("SQ_WAVES", 0.0)
                if not w:
                    continue
                per = lambda c: d.get(c, 0.0) / w
                act = d.get("SQ_LDS_IDX_ACTIVE", 0.0)
                f.write("%-46s %6d %8.0f %8.0f %7.0f %7.0f %7.0f %7.0f %9.1f %14.1f\n" % (
                    k, n[k], w, per("SQ_INSTS_VALU"), per("SQ_INSTS_VALU_TRANS_F32"), per("SQ_INSTS_SALU"), per("SQ_INSTS_LDS"),
                    per("SQ_INSTS_VMEM"), d.get("SQ_INSTS_VALU", 0.0) * 4 / (SIMDS * 2.4e9) * 1e6,
                    100.0 * d.get("SQ_LDS_BANK_CONFLICT", 0.0) / act if act else 0.0))


if __name__ == "__main__":
    main()
