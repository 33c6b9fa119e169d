#!/usr/bin/env python3
"""Condense rocprofv3 CSV output into the short text summaries kept under profiles/.

  rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o p -- python3 bench.py ...
  python3 -m paper_1802_09723_amd.rocprof_summary DIR            # per-kernel durations

  rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR -o p -- python3 bench.py ...
  python3 -m paper_1802_09723_amd.rocprof_summary DIR            # + per-dispatch counter averages

Kernels are grouped by (name, grid, workgroup) because one templated kernel serves several
layers.  Counter rows give the mean value per dispatch.  With --copy-bytes N the dispatches of the
plain copy the benchmark runs for calibration (a torch elementwise kernel moving N bytes each
way) are used to turn FETCH_SIZE / WRITE_SIZE readings into bytes: scale = N / reading(copy).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os
import re
import sys


def short(name: str) -> str:
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    name = name.replace("void ", "").replace("rrm::", "")
    m = re.match(r"([\w:]+)(<[^(]*>)?", name)
    if not m:
        return name[:60]
    base, targs = m.group(1), m.group(2) or ""
    if len(targs) > 28:
        targs = targs[:25] + "...>"
    return (base + targs)[:64]


def find(d: str, suffix: str):
    f = sorted(glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True))
    return f[0] if f else None


def kernel_table(path: str):
    groups = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        wg = int(r["Workgroup_Size_X"]) * int(r["Workgroup_Size_Y"]) * int(r["Workgroup_Size_Z"])
        grid = (int(r["Grid_Size_X"]) // max(1, int(r["Workgroup_Size_X"])),
                int(r["Grid_Size_Y"]) // max(1, int(r["Workgroup_Size_Y"])),
                int(r["Grid_Size_Z"]) // max(1, int(r["Workgroup_Size_Z"])))
        key = (short(r["Kernel_Name"]), grid, wg)
        g = groups.setdefault(key, {"n": 0, "sum": 0.0, "min": 1e30, "max": 0.0,
                                    "vgpr": r["VGPR_Count"], "lds": r["LDS_Block_Size"]})
        dt = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1000.0
        g["n"] += 1
        g["sum"] += dt
        g["min"] = min(g["min"], dt)
        g["max"] = max(g["max"], dt)
    return groups


def counter_table(path: str):
    acc = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        key = (short(r["Kernel_Name"]), int(r["Grid_Size"]) // max(1, int(r["Workgroup_Size"])), r["Counter_Name"])
        a = acc.setdefault(key, [0, 0.0])
        a[0] += 1
        a[1] += float(r["Counter_Value"])
    return acc


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("dir")
    ap.add_argument("--copy-bytes", type=int, default=0,
                    help="bytes the calibration copy kernel moves each way per dispatch")
    ap.add_argument("--copy-kernel", default="AUnaryF", help="substring naming the calibration kernel")
    ap.add_argument("--min-calls", type=int, default=1)
    a = ap.parse_args(argv)

    kt = find(a.dir, "kernel_trace.csv")
    if kt:
        groups = kernel_table(kt)
        total = sum(g["sum"] for g in groups.values())
        print("kernel (grid in workgroups, workgroup size)                                   calls   avg us   min us   max us  share  vgpr    lds")
        for (name, grid, wg), g in sorted(groups.items(), key=lambda kv: -kv[1]["sum"]):
            if g["n"] < a.min_calls:
                continue
            print("%-64s %-18s %6d %8.2f %8.2f %8.2f %5.1f%% %5s %6s" % (
                name, "%dx%dx%d/%d" % (grid + (wg,)), g["n"], g["sum"] / g["n"], g["min"], g["max"],
                100.0 * g["sum"] / total, g["vgpr"], g["lds"]))
    cc = find(a.dir, "counter_collection.csv")
    if cc:
        acc = counter_table(cc)
        scale = {}
        if a.copy_bytes:
            best = {}
            for (name, wgs, ctr), (n, s) in acc.items():  # the copy is the largest launch of that name
                if a.copy_kernel in name and wgs > best.get(ctr, (0, 0, 0))[0]:
                    best[ctr] = (wgs, n, s)
            for ctr, (wgs, n, s) in best.items():
                if s > 0:
                    scale[ctr] = a.copy_bytes / (s / n)
                    print("calibration: %s reads %.1f per copy dispatch of %d bytes -> %.2f bytes per count" % (
                        ctr, s / n, a.copy_bytes, scale[ctr]))
        print("kernel (workgroups)                                                       counter            dispatches   mean/dispatch      bytes")
        for (name, wgs, ctr), (n, s) in acc.items():
            if n < a.min_calls:
                continue
            b = ("%12.0f" % (scale[ctr] * s / n)) if ctr in scale else "           -"
            print("%-64s %-8d %-18s %8d %15.1f %s" % (name, wgs, ctr, n, s / n, b))
    if not kt and not cc:
        print("no rocprofv3 CSV output under", a.dir, file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
