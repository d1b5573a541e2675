"""Condenses rocprofv3 output of ``bench.py`` runs into the short summaries kept under ``profiles/``.

Inputs are the output directories of separate rocprofv3 runs of the same command (rocprofv3 does not
split counters over passes, so every counter set gets a run of its own):

    rocprofv3 --kernel-trace --stats --output-format csv -d <trace> -- python3 bench.py --workload K --steps-only
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <fetch> -- python3 bench.py --workload K --steps-only
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <write> -- python3 bench.py --workload K --steps-only
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <cfetch> -- python3 bench.py --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <cwrite> -- python3 bench.py --calibrate-copy

    python -m paper_2403_07339_amd.profile_summary --workload K --trace <trace> --fetch <fetch> --write <write> \
        --calib-fetch <cfetch> --calib-write <cwrite> --out profiles/bench_workloadK_kernels

writes ``<out>.json`` (what ``bench.py`` reads its ``traffic`` figures from) and ``<out>.md``.  The traffic
counters are in KiB per dispatch; each is scaled by what the same counter reads for a plain copy kernel of
known size (``--calibrate-copy``: 1 GiB read and 1 GiB written per launch).  No arithmetic of the method
lives here: this only reads profiler tables.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re

CALIB_BYTES = 1 << 30  # bytes read and bytes written per launch of the --calibrate-copy kernel


def _find(directory: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not hits:
        raise FileNotFoundError(f"no *{suffix} under {directory}")
    return hits[-1]


def short_name(name: str) -> str:
    """``void imu::gemm_i8_kernel<0>(imu::GemmArgs)`` -> ``gemm_i8_kernel<0>``."""
    name = re.sub(r"^void\s+", "", name)
    name = name.split("(")[0]
    return name.replace("imu::", "")


def read_trace(directory: str):
    rows = collections.defaultdict(list)
    with open(_find(directory, "_kernel_trace.csv")) as f:
        for r in csv.DictReader(f):
            grid = int(r["Grid_Size_X"]) * int(r.get("Grid_Size_Y", 1) or 1) * int(r.get("Grid_Size_Z", 1) or 1)
            rows[(short_name(r["Kernel_Name"]), grid)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    return rows


def read_counter(directory: str, counter: str):
    rows = collections.defaultdict(list)
    with open(_find(directory, "_counter_collection.csv")) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                rows[(short_name(r["Kernel_Name"]), int(r["Grid_Size"]))].append(float(r["Counter_Value"]))
    return rows


def calibration(directory: str, counter: str) -> float:
    """Bytes per counter unit: the largest launches of the calibration run are the 1 GiB copies."""
    rows = read_counter(directory, counter)
    best = max(rows.items(), key=lambda kv: (sum(kv[1]) / len(kv[1])) if "elementwise" in kv[0][0] else -1.0)
    mean = sum(best[1]) / len(best[1])
    return CALIB_BYTES / mean


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, required=True)
    ap.add_argument("--trace", required=True)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--calib-fetch")
    ap.add_argument("--calib-write")
    ap.add_argument("--out", required=True)
    ap.add_argument("--command", default="python3 bench.py --workload K --steps-only")
    args = ap.parse_args()

    trace = read_trace(args.trace)
    fetch = read_counter(args.fetch, "FETCH_SIZE") if args.fetch else {}
    write = read_counter(args.write, "WRITE_SIZE") if args.write else {}
    f_scale = calibration(args.calib_fetch, "FETCH_SIZE") if args.calib_fetch else None
    w_scale = calibration(args.calib_write, "WRITE_SIZE") if args.calib_write else None

    kernels = []
    total_us = sum(sum(v) for v in trace.values())
    for (name, grid), durs in sorted(trace.items(), key=lambda kv: -sum(kv[1])):
        if not (name.startswith(("gemm", "scatter", "qscan", "fixup", "bound", "greedy", "layouts", "level_major",
                                 "setup", "ob_copy", "zero_lists", "identity", "recombine", "select", "reset"))):
            continue
        row = {"kernel": name, "grid_threads": grid, "launches": len(durs), "avg_us": sum(durs) / len(durs),
               "min_us": min(durs), "max_us": max(durs), "share_of_gpu_time": sum(durs) / total_us}
        for key, table, scale in (("hbm_read_bytes", fetch, f_scale), ("hbm_written_bytes", write, w_scale)):
            vals = table.get((name, grid))
            row[key] = (sum(vals) / len(vals)) * scale if vals and scale else None
        kernels.append(row)
    cmd = args.command.replace("--workload K", f"--workload {args.workload}")
    doc = {"workload": args.workload, "command": cmd,
           "calibration": {"FETCH_SIZE_bytes_per_unit": f_scale, "WRITE_SIZE_bytes_per_unit": w_scale,
                           "copy_bytes_per_launch": CALIB_BYTES},
           "kernels": kernels}
    with open(args.out + ".json", "w") as f:
        json.dump(doc, f, indent=1)
        f.write("\n")
    with open(args.out + ".md", "w") as f:
        f.write(f"# rocprofv3: bench.py, workload {args.workload}, the kernels of the timed step\n\n")
        f.write("Commands (on the MI355X box, `cd /tmp && export TMPDIR=/tmp` first; one rocprofv3 run per line):\n\n")
        f.write(f"    rocprofv3 --kernel-trace --stats --output-format csv -d <trace> -- {cmd}\n")
        f.write(f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <fetch> -- {cmd}\n")
        f.write(f"    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <write> -- {cmd}\n")
        f.write("    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <cfetch> -- python3 bench.py --calibrate-copy\n")
        f.write("    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <cwrite> -- python3 bench.py --calibrate-copy\n")
        f.write(f"    python -m paper_2403_07339_amd.profile_summary --workload {args.workload} --trace <trace> --fetch <fetch> "
                "--write <write> --calib-fetch <cfetch> --calib-write <cwrite> --out " + args.out + "\n\n")
        if f_scale and w_scale:
            f.write(f"Traffic counters are KiB per dispatch, scaled by a plain copy of 1 GiB: FETCH_SIZE counts "
                    f"{f_scale:.1f} bytes per unit, WRITE_SIZE {w_scale:.1f}.\n\n")
        f.write("Per launch, mean over the launches of the run (durations from the dispatch records of the kernel trace):\n\n")
        f.write("| kernel | grid (threads) | launches | avg us | min us | max us | % of GPU time | HBM read MB | HBM written MB |\n")
        f.write("|---|---:|---:|---:|---:|---:|---:|---:|---:|\n")
        for r in kernels:
            rd = "-" if r["hbm_read_bytes"] is None else f"{r['hbm_read_bytes'] / 1e6:.1f}"
            wr = "-" if r["hbm_written_bytes"] is None else f"{r['hbm_written_bytes'] / 1e6:.1f}"
            f.write(f"| {r['kernel']} | {r['grid_threads']} | {r['launches']} | {r['avg_us']:.1f} | {r['min_us']:.1f} | "
                    f"{r['max_us']:.1f} | {100 * r['share_of_gpu_time']:.1f} | {rd} | {wr} |\n")
    print(f"wrote {args.out}.json and {args.out}.md ({len(kernels)} kernels)")


if __name__ == "__main__":
    main()
