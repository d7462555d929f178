#!/usr/bin/env python3
"""Condense rocprofv3 CSV output into a short text table.

    python3 paper_2509_24007_amd/profile_summary.py <rocprofv3 output dir> [--min-calls N]

Reads *_kernel_trace.csv (per-dispatch start/end timestamps) and/or *_counter_collection.csv (per-dispatch counter
values) below the directory and groups dispatches by (kernel name, grid size, workgroup size): launches of one
kernel from the decode loop share a grid and so form one group, apart from the prefill launches of the same kernel.
"""
import collections
import csv
import glob
import sys


def short(name):
    name = name.replace("void ", "").replace("sdlm::", "")
    cut = name.find("(")
    return (name if cut < 0 else name[:cut])[:64]


def main():
    d = sys.argv[1]
    min_calls = int(sys.argv[sys.argv.index("--min-calls") + 1]) if "--min-calls" in sys.argv else 8
    dur = collections.defaultdict(list)
    for f in glob.glob(d + "/**/*kernel_trace.csv", recursive=True):
        for r in csv.DictReader(open(f)):
            key = (short(r["Kernel_Name"]), r.get("Grid_Size", r.get("Grid_Size_X", "?")), r.get("Workgroup_Size", r.get("Workgroup_Size_X", "?")))
            dur[key].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    if dur:
        total = sum(sum(v) for v in dur.values())
        print("%-64s %10s %6s %8s %10s %10s %10s %7s" % ("kernel", "grid", "wg", "calls", "avg_us", "min_us", "max_us", "time%"))
        for key, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
            if len(v) < min_calls:
                continue
            print("%-64s %10s %6s %8d %10.2f %10.2f %10.2f %7.2f" % (key[0], key[1], key[2], len(v), sum(v) / len(v), min(v), max(v), 100 * sum(v) / total))
    cnt = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in glob.glob(d + "/**/*counter_collection.csv", recursive=True):
        for r in csv.DictReader(open(f)):
            key = (short(r["Kernel_Name"]), r["Grid_Size"], r["Workgroup_Size"])
            cnt[key][r["Counter_Name"]].append(float(r["Counter_Value"]))
    if cnt:
        print("%-64s %10s %6s %8s  %s" % ("kernel", "grid", "wg", "calls", "counter: mean per dispatch"))
        for key, cs in sorted(cnt.items(), key=lambda kv: -len(next(iter(kv[1].values())))):
            n = len(next(iter(cs.values())))
            if n < min_calls:
                continue
            print("%-64s %10s %6s %8d  %s" % (key[0], key[1], key[2], n, "  ".join("%s=%.6g" % (c, sum(v) / len(v)) for c, v in sorted(cs.items()))))


if __name__ == "__main__":
    main()
