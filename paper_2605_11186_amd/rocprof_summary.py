"""Text summaries of rocprofv3 output for this library's kernels.

    python -m paper_2605_11186_amd.rocprof_summary kernel-trace RESULTS.db
    python -m paper_2605_11186_amd.rocprof_summary traffic FETCH.csv WRITE.csv

`kernel-trace` reads the database that `rocprofv3 --kernel-trace --stats -d DIR -o NAME -- CMD`
leaves behind and prints calls / total / average / min / max duration per kernel (dispatch end -
dispatch begin).  `traffic` reads the counter_collection.csv files of two runs of the same command,
one with `--pmc FETCH_SIZE` and one with `--pmc WRITE_SIZE` (`--output-format csv`), scales both
counters by what they read for a plain copy kernel of known size in the same run
(`bench.py --calibrate-copy`: one 1 GiB device-to-device copy) and prints the HBM bytes per
dispatch for every kernel, per launch of the weight-streaming GEMM, and per verify step (all
`cats_*` kernels of one step; steps are counted by the one `cats_accept` dispatch each has).
Nothing here touches a GPU: it only reads files.
"""
from __future__ import annotations

import argparse
import collections
import csv
import re
import sqlite3

COPY_KIB = 1 << 20   # the calibration copy moves 1 GiB each way


def _short(name: str) -> str:
    return re.sub(r"\(anonymous namespace\)::", "", name)


def kernel_trace(db_path: str) -> str:
    con = sqlite3.connect(db_path)
    rows = con.execute("select name, count(*), sum(end-start), avg(end-start), min(end-start), max(end-start) "
                       "from kernels group by name order by 3 desc").fetchall()
    total = sum(r[2] for r in rows)
    out = [f"{'kernel':72s} {'calls':>6s} {'total_ms':>10s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}"]
    for name, calls, tot, avg, mn, mx in rows:
        out.append(f"{_short(name)[:72]:72s} {calls:6d} {tot / 1e6:10.3f} {avg / 1e3:9.2f} {mn / 1e3:9.2f} "
                   f"{mx / 1e3:9.2f} {100 * tot / total:6.2f}")
    out.append(f"total kernel time {total / 1e6:.3f} ms")
    steps = sum(r[1] for r in rows if "cats_accept(" in r[0])
    if steps:
        step_ns = sum(r[2] for r in rows if "cats_" in r[0] and "pack_matrix" not in r[0])
        out.append(f"{steps} verify steps in the trace; kernel time of the step's own kernels (cats_*, without the "
                   f"one-time weight re-tiling): {step_ns / steps / 1e6:.3f} ms per step")
    return "\n".join(out)


def _per_kernel(csv_path: str):
    d = collections.defaultdict(list)
    with open(csv_path) as f:
        for row in csv.DictReader(f):
            d[row["Kernel_Name"]].append(float(row["Counter_Value"]))
    return d


def traffic(fetch_csv: str, write_csv: str) -> str:
    fetch, write = _per_kernel(fetch_csv), _per_kernel(write_csv)
    copy = [k for k in fetch if "copyBuffer" in k]
    if not copy:
        raise SystemExit("no copy kernel in the run: pass --calibrate-copy to bench.py")
    f_copy, w_copy = max(fetch[copy[0]]), max(write[copy[0]])
    f_scale, w_scale = COPY_KIB / f_copy, COPY_KIB / w_copy
    mean = lambda v: sum(v) / len(v) if v else 0.0
    steps = len(fetch.get(next((k for k in fetch if "cats_accept(" in k), ""), []))
    out = ["calibration: one 1 GiB device-to-device copy (reads 1048576 KiB, writes 1048576 KiB)",
           f"  copy kernel {copy[0]}: FETCH_SIZE = {f_copy:.1f}, WRITE_SIZE = {w_copy:.1f}",
           f"  => scale factors: fetch x{f_scale:.4f}, write x{w_scale:.4f} (counter units -> KiB)",
           "",
           f"{'kernel (mean per dispatch)':64s} {'dispatches':>10s} {'per step':>9s} {'read MB':>9s} {'written MB':>11s}"]
    step_bytes = 0.0
    gemm = None
    for k in sorted(fetch, key=lambda k: -mean(fetch[k]) * len(fetch[k])):
        if "cats_" not in k:
            continue
        rd = mean(fetch[k]) * f_scale * 1024
        wr = mean(write.get(k, [])) * w_scale * 1024
        n = len(fetch[k])
        per_step = n / steps if steps else 0.0
        out.append(f"{_short(k)[:64]:64s} {n:10d} {per_step:9.1f} {rd / 1e6:9.2f} {wr / 1e6:11.2f}")
        if "pack_matrix" not in k:
            step_bytes += (rd + wr) * per_step
        if "cats_gemm" in k:
            gemm = (rd, wr)
    out.append("")
    if gemm:
        out.append(f"GEMM: {gemm[0] / 1e6:.1f} MB read + {gemm[1] / 1e6:.1f} MB written per launch")
        out.append(f"gemm_traffic_bytes_per_launch: {int(gemm[0] + gemm[1])}")
    if steps:
        out.append(f"{steps} verify steps in the run; all cats_* kernels of one step (without the one-time weight re-tiling):")
        out.append(f"step_traffic_bytes: {int(step_bytes)}")
    return "\n".join(out)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    kt = sub.add_parser("kernel-trace")
    kt.add_argument("db")
    tr = sub.add_parser("traffic")
    tr.add_argument("fetch_csv")
    tr.add_argument("write_csv")
    args = ap.parse_args()
    print(kernel_trace(args.db) if args.what == "kernel-trace" else traffic(args.fetch_csv, args.write_csv))


if __name__ == "__main__":
    main()
