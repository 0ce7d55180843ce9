#!/usr/bin/env python3
"""Turns the csv files of three rocprofv3 runs of one bench.py command into the short summary kept under
profiles/ (markdown on stdout) and, for the headline kernel, the small json that bench.py reads its measured
HBM traffic from.

The three runs (from /tmp with TMPDIR=/tmp, the program directly after `--`), all into one directory D:

    rocprofv3 --kernel-trace --stats --output-format csv -d D -o kt    -- python3 bench.py ...
    rocprofv3 --pmc FETCH_SIZE       --output-format csv -d D -o fetch -- python3 bench.py ...
    rocprofv3 --pmc WRITE_SIZE       --output-format csv -d D -o write -- python3 bench.py ...

    python3 bench_profile.py D --kernels k_copy_sweep_stream [--per-dispatch] [--json profiles/X_traffic.json --commit HASH]

FETCH_SIZE / WRITE_SIZE are reported per dispatch in units that are scaled here by what the same counter reads for
a plain copy of known size in the same run: the largest dispatch of the calibration kernel (a 1 GiB tensor copy,
`--calibration-copy` or any `--profile-cells` mode of bench.py).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import sys


def find(d, tag, kind):
    hits = sorted(glob.glob(os.path.join(d, "**", f"{tag}_{kind}.csv"), recursive=True))
    return hits[-1] if hits else None


def short(name):
    return name.split("(")[0].replace("void ", "").replace("shmemx::", "")[:64]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("dir")
    ap.add_argument("--kernels", default="k_", help="comma list of substrings: kernels to report counters for")
    ap.add_argument("--calib", default="copyBuffer", help="substring of the calibration kernel's name")
    ap.add_argument("--calib-bytes", type=float, default=float(1 << 30), help="bytes the calibration copy reads (and writes)")
    ap.add_argument("--per-dispatch", action="store_true", help="list counters dispatch by dispatch (launch order)")
    ap.add_argument("--json", default=None, help="write the traffic of the FIRST kernel of --kernels to this file")
    ap.add_argument("--commit", default=None)
    ap.add_argument("--command", default=None)
    args = ap.parse_args()
    pats = [p for p in args.kernels.split(",") if p]

    stats = find(args.dir, "kt", "kernel_stats")
    if stats:
        print("## Kernel trace (--stats)\n")
        print("| kernel | calls | total ms | avg us | min us | max us | % |\n|---|---|---|---|---|---|---|")
        for r in list(csv.DictReader(open(stats)))[:10]:
            print(f"| {short(r['Name'])} | {r['Calls']} | {float(r['TotalDurationNs']) / 1e6:.3f} | {float(r['AverageNs']) / 1e3:.2f} | "
                  f"{float(r['MinNs']) / 1e3:.2f} | {float(r['MaxNs']) / 1e3:.2f} | {float(r['Percentage']):.2f} |")
        print()

    per = {}          # tag -> kernel -> [(dispatch, value)]
    for tag, counter in (("fetch", "FETCH_SIZE"), ("write", "WRITE_SIZE")):
        f = find(args.dir, tag, "counter_collection")
        if not f:
            continue
        by = collections.defaultdict(dict)
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] != counter:
                continue
            key = (short(r["Kernel_Name"]), int(r["Dispatch_Id"]))
            by[key[0]][key[1]] = by[key[0]].get(key[1], 0.0) + float(r["Counter_Value"])
        per[tag] = {k: sorted(v.items()) for k, v in by.items()}
    if not per:
        return
    scale = {}
    print("## HBM traffic counters (--pmc), scaled by the plain copy of the same run\n")
    for tag in ("fetch", "write"):
        cal = [v for k, rows in per.get(tag, {}).items() if args.calib in k for _, v in rows]
        if not cal:
            print(f"- no calibration dispatch ({args.calib}) in the {tag} run: raw counter units below")
            scale[tag] = None
            continue
        scale[tag] = args.calib_bytes / max(cal)
        print(f"- {tag}: the {args.calib_bytes / (1 << 30):.0f} GiB copy reads {max(cal):.1f} counter units -> {scale[tag]:.1f} bytes per unit")
    print()
    report = {}
    for tag in ("fetch", "write"):
        for k, rows in per.get(tag, {}).items():
            if not any(p in k for p in pats):
                continue
            sc = scale.get(tag) or 1.0
            report.setdefault(k, {})[tag] = [(d, v * sc) for d, v in rows]
    print("| kernel | dispatches | fetched per dispatch | written per dispatch | total |\n|---|---|---|---|---|")
    for k, t in report.items():
        fe = [v for _, v in t.get("fetch", [])]
        wr = [v for _, v in t.get("write", [])]
        fa, wa = (sum(fe) / len(fe) if fe else 0.0), (sum(wr) / len(wr) if wr else 0.0)
        print(f"| {k} | {max(len(fe), len(wr))} | {fa / 1e6:.2f} MB | {wa / 1e6:.2f} MB | {(fa + wa) / 1e6:.2f} MB |")
    if args.per_dispatch:
        print("\nDispatch by dispatch (launch order), MB fetched / written:\n")
        for k, t in report.items():
            fe, wr = t.get("fetch", []), t.get("write", [])
            print(f"- {k}: " + ", ".join(f"{f[1] / 1e6:.1f} / {w[1] / 1e6:.1f}" for f, w in zip(fe, wr)))
    if args.json and pats:
        k = next((k for k in report if pats[0] in k), None)
        if k is None:
            sys.exit(f"no kernel matching {pats[0]} in the counter runs")
        fe = [v for _, v in report[k].get("fetch", [])]
        wr = [v for _, v in report[k].get("write", [])]
        fa, wa = sum(fe) / len(fe), sum(wr) / len(wr)
        with open(args.json, "w") as f:
            json.dump({"kernel": k, "dispatches": len(fe), "fetch_bytes_per_launch": round(fa), "write_bytes_per_launch": round(wa),
                       "traffic_bytes_per_launch": round(fa + wa), "bytes_per_fetch_unit": scale.get("fetch"),
                       "bytes_per_write_unit": scale.get("write"), "commit": args.commit, "command": args.command}, f, indent=1)
            f.write("\n")


if __name__ == "__main__":
    main()
