"""Turns rocprofv3 CSV output into the short text summaries kept under ``profiles/``.

    python -m paper_2203_09044_amd.profiling kernel-stats <dir with *_kernel_stats.csv> --command "<cmd>"
    python -m paper_2203_09044_amd.profiling traffic --fetch <dir> --write <dir> --cal-fetch <dir> --cal-write <dir>
           --kernel k_convert_ef --command "<cmd>" [--json out.json]

``traffic`` scales the FETCH_SIZE / WRITE_SIZE readings of one kernel by what the same counters read for
a plain elementwise copy of known size (``bench.py --calibrate-copy``: 2^30 bytes read, 2^30 written).
"""
from __future__ import annotations

import argparse
import csv
import glob
import json
import os
import re
import sys
from collections import defaultdict

CAL_BYTES = 1 << 30


def _one(pattern_dir, suffix):
    hits = glob.glob(os.path.join(pattern_dir, "**", f"*{suffix}"), recursive=True)
    if not hits:
        raise SystemExit(f"no *{suffix} under {pattern_dir}")
    return hits[0]


def short(name: str) -> str:
    m = re.search(r"\b(k_[a-z0-9_]+)(<[^>]*>)?", name)
    return (m.group(1) + (m.group(2) or "")) if m else name[:60]


def kernel_stats(args):
    rows = [r for r in csv.DictReader(open(_one(args.dir, "_kernel_stats.csv")))]
    ours = [r for r in rows if re.search(r"\bk_[a-z0-9_]+", r["Name"])]
    total = sum(float(r["TotalDurationNs"]) for r in ours)
    print(f"# rocprofv3 --kernel-trace --stats, kernels of libco3 only (torch's input-generation kernels omitted)")
    for line in args.command.split(";"):
        print(f"# command: {line.strip()}")
    print(f"{'kernel':24s} {'calls':>6s} {'avg us':>10s} {'min us':>10s} {'max us':>10s} {'share of path':>14s}")
    for r in sorted(ours, key=lambda r: -float(r["TotalDurationNs"])):
        print(f"{short(r['Name']):24s} {int(r['Calls']):6d} {float(r['AverageNs']) / 1e3:10.2f} "
              f"{float(r['MinNs']) / 1e3:10.2f} {float(r['MaxNs']) / 1e3:10.2f} "
              f"{100 * float(r['TotalDurationNs']) / total:13.1f}%")
    calls = max(int(r["Calls"]) for r in ours)
    print(f"# sum of libco3 kernel time per step: {total / calls / 1e3:.1f} us ({calls} steps incl. warm-up)")


def _counter_avg(d, counter, match):
    vals = defaultdict(list)
    for r in csv.DictReader(open(_one(d, "_counter_collection.csv"))):
        if r["Counter_Name"] == counter:
            vals[short(r["Kernel_Name"]) if "k_" in r["Kernel_Name"] else r["Kernel_Name"]].append(
                float(r["Counter_Value"]))
    out = {k: sum(v) / len(v) for k, v in vals.items() if match(k)}
    return out


def traffic(args):
    cal_f = _counter_avg(args.cal_fetch, "FETCH_SIZE", lambda k: "CUDAFunctorOnSelf_add" in k or "add" in k.lower())
    cal_w = _counter_avg(args.cal_write, "WRITE_SIZE", lambda k: "CUDAFunctorOnSelf_add" in k or "add" in k.lower())
    if not cal_f or not cal_w:
        raise SystemExit("calibration kernel not found")
    f_read = max(cal_f.values())       # counter reading for CAL_BYTES fetched
    w_read = max(cal_w.values())
    f_scale = CAL_BYTES / f_read       # bytes per counter unit
    w_scale = CAL_BYTES / w_read
    fetch = _counter_avg(args.fetch, "FETCH_SIZE", lambda k: k.startswith("k_"))
    write = _counter_avg(args.write, "WRITE_SIZE", lambda k: k.startswith("k_"))
    print("# rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (one run each), per launch, scaled by the readings of a")
    print(f"# plain 1 GiB elementwise copy: FETCH_SIZE {f_read:.0f} -> x{f_scale / 1024:.3f} KiB per unit, "
          f"WRITE_SIZE {w_read:.0f} -> x{w_scale / 1024:.3f} KiB per unit")
    for line in args.command.split(";"):
        print(f"# command: {line.strip()}")
    print(f"{'kernel':24s} {'fetched MB':>12s} {'written MB':>12s} {'total MB':>10s}")
    res = {}
    for k in sorted(set(fetch) | set(write), key=lambda k: -(fetch.get(k, 0) * f_scale + write.get(k, 0) * w_scale)):
        fb, wb = fetch.get(k, 0.0) * f_scale, write.get(k, 0.0) * w_scale
        res[k] = {"fetch_bytes": fb, "write_bytes": wb}
        print(f"{k:24s} {fb / 1e6:12.1f} {wb / 1e6:12.1f} {(fb + wb) / 1e6:10.1f}")
    if args.json:
        key = next((k for k in res if k.startswith(args.kernel)), None)
        if key is None:
            raise SystemExit(f"kernel {args.kernel} not in the counter files")
        json.dump({"kernel": key, "traffic_bytes_per_launch": res[key]["fetch_bytes"] + res[key]["write_bytes"],
                   "fetch_bytes": res[key]["fetch_bytes"], "write_bytes": res[key]["write_bytes"],
                   "fetch_scale": f_scale / 1024, "write_scale": w_scale / 1024, "command": args.command},
                  open(args.json, "w"), indent=1)


def main(argv=None):
    ap = argparse.ArgumentParser(prog="python -m paper_2203_09044_amd.profiling")
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("kernel-stats")
    a.add_argument("dir")
    a.add_argument("--command", default="")
    a.set_defaults(fn=kernel_stats)
    b = sub.add_parser("traffic")
    for o in ("--fetch", "--write", "--cal-fetch", "--cal-write"):
        b.add_argument(o, required=True)
    b.add_argument("--kernel", default="k_convert_ef")
    b.add_argument("--command", default="")
    b.add_argument("--json", default=None)
    b.set_defaults(fn=traffic)
    args = ap.parse_args(argv)
    args.fn(args)


if __name__ == "__main__":
    sys.exit(main())
