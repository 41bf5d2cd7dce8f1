"""Summarises two rocprofv3 counter runs of bench.py (FETCH_SIZE, then WRITE_SIZE) into
HBM-side bytes per launch for every kernel of the library: profiles/traffic_<workload>.json
(read by bench.py for roofline.traffic) and a small table beside it.

The two runs (on the GPU machine, each a run of its own; rocprofv3 writes
<dir>/p_counter_collection.csv):

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir_f> -o p -- \\
        python3 bench.py --workload <w> --steps 1 --warmup 0 --no-cpu-baseline --no-calib --calib-copy-mib 1024
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir_w> -o p -- (the same command)

then, anywhere:

    python -m paper_1606_04884_amd.profsum --fetch <dir_f>/p_counter_collection.csv \\
        --write <dir_w>/p_counter_collection.csv --workload <w> --out-dir profiles

Scaling: --calib-copy-mib makes bench.py run the library's probe_copy_kernel once over that
many MiB before anything else; what each counter reads for it (a known number of bytes read
and written) gives the bytes per counter unit, which is then applied to every dispatch.
"""
from __future__ import annotations

import argparse
import csv
import json
import os
import re
import time


def short_name(full: str) -> str:
    """mi355conv::wino4_gemm_kernel<2, 2>(...) -> wino4_gemm_kernel"""
    m = re.search(r"mi355conv::(?:\(anonymous namespace\)::)?([A-Za-z0-9_]+)", full)
    return m.group(1) if m else ""


def read_counter(path: str, counter: str):
    per = {}
    order = []
    with open(path, newline="") as fh:
        for row in csv.DictReader(fh):
            if row["Counter_Name"] != counter:
                continue
            name = short_name(row["Kernel_Name"])
            if not name:
                continue
            d = per.setdefault(name, [])
            if not d:
                order.append(name)
            d.append(float(row["Counter_Value"]))
    return per, order


def kernel_stats(stats_csv: str, bench_line: str, workload: str, out_dir: str) -> None:
    """profiles/kernel_stats_<workload>.txt from `rocprofv3 --kernel-trace --stats --output-format csv
    -d <dir> -o s -- python3 bench.py --workload <w> --steps 5 --warmup 2` (<dir>/s_kernel_stats.csv) and
    the JSON line that run printed."""
    rows = []
    with open(stats_csv, newline="") as fh:
        for row in csv.DictReader(fh):
            name = short_name(row["Name"]) or row["Name"][:60]
            rows.append((name, int(row["Calls"]), float(row["TotalDurationNs"]) / 1e6, float(row["AverageNs"]) / 1e3,
                         float(row["Percentage"])))
    merged = {}
    for name, calls, tot, _, pct in rows:            # template instances of one kernel together
        m = merged.setdefault(name, [0, 0.0, 0.0])
        m[0] += calls
        m[1] += tot
        m[2] += pct
    with open(os.path.join(out_dir, "kernel_stats_%s.txt" % workload), "w") as fh:
        fh.write("rocprofv3 --kernel-trace --stats summary, %s workload, %s\n" % (workload, time.strftime("%Y-%m-%d")))
        fh.write("command: rocprofv3 --kernel-trace --stats --output-format csv -d out -o s -- python3 bench.py "
                 "--workload %s --steps 5 --warmup 2   (2 warm-up + 5 timed + 5 profiled steps and the probes, "
                 "every launch counted)\nsummarised by: python -m paper_1606_04884_amd.profsum --stats ...\n\n" % workload)
        fh.write("%-64s %8s %12s %12s %7s\n" % ("kernel", "calls", "total_ms", "avg_us", "pct"))
        for name, (calls, tot, pct) in sorted(merged.items(), key=lambda kv: -kv[1][1]):
            fh.write("%-64s %8d %12.3f %12.1f %7.2f\n" % (name, calls, tot, tot * 1e3 / calls, pct))
        fh.write("\nbench.py line of the same run:\n%s\n" % bench_line.strip())


def mfma_util(counter_csv: str, workload: str, out_dir: str) -> None:
    """profiles/mfma_util_<workload>.txt from one counter run with SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_MFMA
    SQ_INSTS_VALU SQ_WAIT_INST_ANY GRBM_GUI_ACTIVE (and others, ignored) collected together."""
    import collections
    per = collections.defaultdict(lambda: collections.defaultdict(float))
    launches = collections.Counter()
    seen = set()
    with open(counter_csv, newline="") as fh:
        for row in csv.DictReader(fh):
            name = short_name(row["Kernel_Name"])
            if not name:
                continue
            per[name][row["Counter_Name"]] += float(row["Counter_Value"])
            if row["Dispatch_Id"] not in seen:
                seen.add(row["Dispatch_Id"])
                launches[name] += 1
    with open(os.path.join(out_dir, "mfma_util_%s.txt" % workload), "w") as fh:
        fh.write("MFMA utilisation per kernel, %s workload, %s (rocprofv3 counters, two passes of the stack)\n" % (
            workload, time.strftime("%Y-%m-%d")))
        fh.write("command: rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_MFMA SQ_BUSY_CYCLES SQ_INSTS_VALU "
                 "SQ_ACTIVE_INST_VALU SQ_WAIT_INST_ANY SQ_WAVE_CYCLES GRBM_GUI_ACTIVE --output-format csv -d out -o u -- "
                 "python3 bench.py --workload %s --steps 1 --warmup 0 --no-cpu-baseline --no-calib\n" % workload)
        fh.write("summarised by: python -m paper_1606_04884_amd.profsum --util <out>/u_counter_collection.csv\n\n")
        fh.write("util = SQ_VALU_MFMA_BUSY_CYCLES / (cycles x 256 compute units x 4 SIMDs), cycles = GRBM_GUI_ACTIVE / 8 (the\n"
                 "counter comes back summed over the 8 XCDs); SQ_VALU_MFMA_BUSY_CYCLES is 64 per v_mfma_f32_32x32x2_f32, so util\n"
                 "is the share of the fp32 matrix pipe's cycles the kernel's MFMAs fill at the clock it actually ran at.\n"
                 "INSTS_VALU counts the MFMAs too: (INSTS_VALU - INSTS_MFMA) / INSTS_MFMA = other vector instructions per MFMA.\n\n")
        fh.write("%-28s %8s %12s %12s %12s %7s %12s %14s\n" % ("kernel", "launches", "GUI_ACTIVE", "MFMA_BUSY", "INSTS_MFMA",
                                                              "util %", "INSTS_VALU", "other per MFMA"))
        for name, c in sorted(per.items(), key=lambda kv: -kv[1]["GRBM_GUI_ACTIVE"]):
            cyc = c["GRBM_GUI_ACTIVE"] / 8.0
            util = 100.0 * c["SQ_VALU_MFMA_BUSY_CYCLES"] / (cyc * 256 * 4) if cyc else 0.0
            other = (c["SQ_INSTS_VALU"] - c["SQ_INSTS_MFMA"]) / c["SQ_INSTS_MFMA"] if c["SQ_INSTS_MFMA"] else float("nan")
            fh.write("%-28s %8d %12.4g %12.4g %12.4g %7.1f %12.4g %14.2f\n" % (
                name, launches[name], c["GRBM_GUI_ACTIVE"], c["SQ_VALU_MFMA_BUSY_CYCLES"], c["SQ_INSTS_MFMA"], util,
                c["SQ_INSTS_VALU"], other))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--stats", help="s_kernel_stats.csv of a --kernel-trace --stats run: write kernel_stats_<workload>.txt")
    ap.add_argument("--bench-line", help="file holding the JSON line that run printed")
    ap.add_argument("--util", help="counter_collection.csv of an MFMA-utilisation counter run: write mfma_util_<workload>.txt")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--workload", required=True)
    ap.add_argument("--calib-mib", type=int, default=1024)
    ap.add_argument("--out-dir", default="profiles")
    args = ap.parse_args()
    if args.util:
        os.makedirs(args.out_dir, exist_ok=True)
        mfma_util(args.util, args.workload, args.out_dir)
        return 0
    if args.stats:
        line = open(args.bench_line).read() if args.bench_line else ""
        os.makedirs(args.out_dir, exist_ok=True)
        kernel_stats(args.stats, line, args.workload, args.out_dir)
        return 0
    if not args.fetch or not args.write:
        raise SystemExit("--fetch and --write (or --stats) are required")

    fetch, order = read_counter(args.fetch, "FETCH_SIZE")
    write, _ = read_counter(args.write, "WRITE_SIZE")
    calib_bytes = float(args.calib_mib) * (1 << 20)
    if "probe_copy_kernel" not in fetch or "probe_copy_kernel" not in write:
        raise SystemExit("no probe_copy_kernel dispatch found: run bench.py with --calib-copy-mib")
    f_unit = calib_bytes / fetch["probe_copy_kernel"][0]
    w_unit = calib_bytes / write["probe_copy_kernel"][0]

    rows = []
    for name in order:
        if name == "probe_copy_kernel" or name not in write:
            continue
        n = len(fetch[name])
        fb = sum(fetch[name]) * f_unit / n
        wb = sum(write[name]) * w_unit / len(write[name])
        rows.append((name, n, fb, wb))
    rows.sort(key=lambda r: -(r[2] + r[3]) * r[1])

    date = time.strftime("%Y-%m-%d")
    out = {
        "workload": args.workload, "date": date,
        "command": "rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE --output-format csv -- python3 bench.py --workload %s --steps 1 "
                   "--warmup 0 --no-cpu-baseline --no-calib --calib-copy-mib %d" % (args.workload, args.calib_mib),
        "bytes_per_counter_unit": {"FETCH_SIZE": round(f_unit, 2), "WRITE_SIZE": round(w_unit, 2)},
        "launches": {r[0]: r[1] for r in rows},
        "fetch_bytes_per_launch": {r[0]: int(r[2]) for r in rows},
        "write_bytes_per_launch": {r[0]: int(r[3]) for r in rows},
        "bytes_per_launch": {r[0]: int(r[2] + r[3]) for r in rows},
    }
    os.makedirs(args.out_dir, exist_ok=True)
    with open(os.path.join(args.out_dir, "traffic_%s.json" % args.workload), "w") as fh:
        json.dump(out, fh, indent=1)
        fh.write("\n")
    with open(os.path.join(args.out_dir, "traffic_%s.md" % args.workload), "w") as fh:
        fh.write("HBM-side traffic per launch, %s workload (one pass of the stack), %s\n\n" % (args.workload, date))
        fh.write("command (two runs, one counter each): %s\n" % out["command"])
        fh.write("summarised by: python -m paper_1606_04884_amd.profsum (this file and traffic_%s.json)\n" % args.workload)
        fh.write("scaling from the probe_copy_kernel dispatch over %d MiB: %.1f bytes per FETCH_SIZE unit, "
                 "%.1f per WRITE_SIZE unit\n\n" % (args.calib_mib, f_unit, w_unit))
        fh.write("| kernel | launches | fetch MB / launch | write MB / launch |\n|---|---|---|---|\n")
        for name, n, fb, wb in rows:
            fh.write("| %s | %d | %.1f | %.1f |\n" % (name, n, fb / 1e6, wb / 1e6))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
