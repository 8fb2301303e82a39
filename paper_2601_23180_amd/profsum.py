"""Per-kernel summary of rocprofv3 CSV output (argument parsing and averaging only).

    python -m paper_2601_23180_amd.profsum DIR [--json OUT]

DIR is searched recursively for `*_kernel_trace.csv` (from `--kernel-trace`) and
`*_counter_collection.csv` (from `--pmc ...`), both written with `--output-format csv`.
Prints, per kernel name: launches, mean duration, and the mean of every collected counter per
dispatch.  With a copy-probe kernel (`k_copy_probe`, bytes read = bytes written = its size) in
the same run, counters that measure memory traffic can be scaled to bytes by the caller.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import sys


def short(name: str) -> str:
    name = re.sub(r"\(.*$", "", name).replace("void ", "").strip()
    return name


def col(row, *names):
    for n in names:
        if n in row and row[n] != "":
            return row[n]
    raise KeyError(names)


def kernel_trace(path):
    agg = collections.OrderedDict()
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            name = short(col(row, "Kernel_Name", "kernel_name", "Name"))
            t0 = int(col(row, "Start_Timestamp", "start_timestamp", "Start"))
            t1 = int(col(row, "End_Timestamp", "end_timestamp", "End"))
            a = agg.setdefault(name, [0, 0])
            a[0] += 1
            a[1] += t1 - t0
    return {k: {"launches": v[0], "avg_us": v[1] / v[0] / 1e3, "total_ms": v[1] / 1e6} for k, v in agg.items()}


def counters(path):
    per = collections.OrderedDict()
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            name = short(col(row, "Kernel_Name", "kernel_name"))
            cname = col(row, "Counter_Name", "counter_name")
            val = float(col(row, "Counter_Value", "counter_value"))
            disp = col(row, "Dispatch_Id", "dispatch_id", "Correlation_Id")
            d = per.setdefault((name, cname), {})
            d[disp] = d.get(disp, 0.0) + val      # one row per (dispatch, counter instance)
    out = collections.OrderedDict()
    for (name, cname), d in per.items():
        out.setdefault(name, {})[cname] = {"dispatches": len(d), "mean_per_dispatch": sum(d.values()) / len(d)}
    return out


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("dir")
    ap.add_argument("--json", default=None)
    args = ap.parse_args(argv)
    res = {"kernel_trace": {}, "counters": {}}
    for p in sorted(glob.glob(os.path.join(args.dir, "**", "*_kernel_trace.csv"), recursive=True)):
        res["kernel_trace"].update(kernel_trace(p))
    for p in sorted(glob.glob(os.path.join(args.dir, "**", "*_counter_collection.csv"), recursive=True)):
        for k, v in counters(p).items():
            res["counters"].setdefault(k, {}).update(v)
    if res["kernel_trace"]:
        tot = sum(v["total_ms"] for v in res["kernel_trace"].values())
        print(f"{'kernel':70s} {'launches':>9s} {'avg us':>10s} {'total ms':>10s} {'%':>6s}")
        for k, v in sorted(res["kernel_trace"].items(), key=lambda kv: -kv[1]["total_ms"]):
            print(f"{k[:70]:70s} {v['launches']:9d} {v['avg_us']:10.2f} {v['total_ms']:10.3f} {100 * v['total_ms'] / tot:6.1f}")
    for k, v in res["counters"].items():
        for c, s in v.items():
            print(f"{k[:70]:70s} {c:16s} dispatches {s['dispatches']:6d}  mean/dispatch {s['mean_per_dispatch']:.6g}")
    if args.json:
        with open(args.json, "w") as f:
            json.dump(res, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
