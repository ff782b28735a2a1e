"""Turns rocprofv3 output of `bench.py` runs into the figures the benchmark line and `profiles/` quote.

rocprofv3 writes one CSV per run (`*_counter_collection.csv` for `--pmc`, `*_kernel_stats.csv` / `*_kernel_trace.csv`
for `--kernel-trace --stats`).  This script reads them, never the GPU:

    python -m paper_2311_09550_amd.counters traffic --fetch DIR --write DIR --kernel NAME --key KEY --calls-per-dispatch F
        HBM-side bytes per GEMM call of the kernel whose name contains NAME: FETCH_SIZE and WRITE_SIZE (KiB-like units
        per dispatch), each scaled by what the same counter reads for the 256 MiB `__amd_rocclr_copyBuffer` dispatches
        of `bench.py --copy-calibration` in the same run, summed over all dispatches of the kernel and divided by the
        GEMM calls of the run = dispatches x F (a GEMM call may be more than one dispatch: the timed step makes 4 calls
        in 5 dispatches, F = 0.8; default F = 1); with --by-grid instead the mean over the GEMM shapes of the mean per
        dispatch (the decode section: a shape is told by grid size and k steps per wave; equal weights).  Merges the result under KEY into
        profiles/traffic_counters.json together with the hash of the kernel sources, which `bench.py` checks before it
        reports the figure.  Prints a markdown table per (kernel, grid size).

    python -m paper_2311_09550_amd.counters sq --dir DIR --kernel NAME
        Means per dispatch of every counter in a `--pmc SQ_...` run, per (kernel, grid size), as a markdown table.

    python -m paper_2311_09550_amd.counters stats --dir DIR
        The library's rows of a `--kernel-trace --stats` run as a markdown table, plus the median / minimum duration
        per (kernel, grid size) from the trace.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import statistics
import sys

from .build import source_hash

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_counters.json")
COPY_KERNEL = "__amd_rocclr_copyBuffer"
COPY_KIB = 256 * 1024   # the calibration copy reads and writes 256 MiB


def _one(pattern_dir, suffix):
    files = glob.glob(os.path.join(pattern_dir, "**", "*" + suffix), recursive=True)
    if not files:
        sys.exit(f"no *{suffix} under {pattern_dir}")
    return files[0]


def _counter_rows(directory):
    with open(_one(directory, "counter_collection.csv")) as f:
        yield from csv.DictReader(f)


def _short(name):
    name = name.replace("void ", "").replace("(anonymous namespace)::", "").replace("w4a8::", "")
    return name.split("(")[0]


def _per_dispatch(directory, counter):
    """[(kernel name, grid size, value)] of one counter, and the mean of the calibration copies."""
    rows, copies = [], []
    for r in _counter_rows(directory):
        if r["Counter_Name"] != counter:
            continue
        v = float(r["Counter_Value"])
        if COPY_KERNEL in r["Kernel_Name"] and v > 1000:
            copies.append(v)
        rows.append((r["Kernel_Name"], int(r["Grid_Size"]), v))
    # other device copies of the run (clones of weight arrays) are smaller than the 256 MiB calibration copy
    copies = [v for v in copies if v >= 0.9 * max(copies)]
    return rows, (sum(copies) / len(copies) if copies else None)


def cmd_traffic(a):
    fetch, fcal = _per_dispatch(a.fetch, "FETCH_SIZE")
    write, wcal = _per_dispatch(a.write, "WRITE_SIZE")
    if fcal is None or wcal is None:
        sys.exit("no calibration copy in the run: profile `bench.py --copy-calibration`")
    fscale, wscale = COPY_KIB / fcal, COPY_KIB / wcal   # counter units -> KiB
    groups = collections.defaultdict(lambda: {"fetch": [], "write": []})
    for rows, what, scale in ((fetch, "fetch", fscale), (write, "write", wscale)):
        for name, grid, v in rows:
            if a.kernel in name:
                groups[(_short(name), grid)][what].append(v * scale * 1024.0)
    if not groups:
        sys.exit(f"no dispatch of a kernel named *{a.kernel}* in the run")
    print(f"Calibration: FETCH_SIZE reads {fcal:.1f} and WRITE_SIZE {wcal:.1f} for the 256 MiB copy "
          f"(262144 KiB read, 262144 KiB written): factors {fscale:.3f} and {wscale:.3f}.\n")
    print("| kernel | grid (threads) | dispatches | fetched MB / dispatch | written MB / dispatch |")
    print("|---|---|---|---|---|")
    total_f = total_w = 0.0
    for (name, grid), g in sorted(groups.items()):
        total_f += sum(g["fetch"])
        total_w += sum(g["write"])
        print(f"| `{name}` | {grid} | {len(g['fetch'])} | {statistics.mean(g['fetch']) / 1e6:.2f} | "
              f"{statistics.mean(g['write']) / 1e6:.2f} |")
    n_f = sum(len(g["fetch"]) for g in groups.values())
    n_w = sum(len(g["write"]) for g in groups.values())
    if n_f != n_w:
        print(f"\n(the two runs saw {n_f} and {n_w} dispatches: each total is divided by its own run's GEMM calls)")
    gemms = n_f * a.calls_per_dispatch
    if a.by_grid:
        # one GEMM shape per (grid size, k steps per wave = second template argument of the kernel): every shape with
        # the same weight, however many launches each had and whichever instantiations served its token counts
        by_grid = collections.defaultdict(lambda: {"fetch": [], "write": []})
        for (name, grid), g in groups.items():
            args = name[name.find("<") + 1:].split(",") if "<" in name else []
            key = (grid, args[1].strip() if len(args) > 1 else "")
            by_grid[key]["fetch"] += g["fetch"]
            by_grid[key]["write"] += g["write"]
        per_f = statistics.mean(statistics.mean(g["fetch"]) for g in by_grid.values())
        per_w = statistics.mean(statistics.mean(g["write"]) for g in by_grid.values())
        print(f"\nPer GEMM call, mean over the {len(by_grid)} GEMM shapes (grid size, k steps per wave) of the mean per dispatch: "
              f"{per_f / 1e6:.2f} MB fetched + {per_w / 1e6:.2f} MB written = {(per_f + per_w) / 1e6:.2f} MB.")
    else:
        per_f, per_w = total_f / gemms, total_w * (n_f / n_w if n_w else 1.0) / gemms
        print(f"\nPer GEMM call ({gemms:.0f} calls in {n_f} dispatches): {per_f / 1e6:.2f} MB fetched + {per_w / 1e6:.2f} MB written = "
              f"{(per_f + per_w) / 1e6:.2f} MB.")
    try:
        prof = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        prof = {}
    h = source_hash()
    if prof.get("source_hash") != h:
        prof = {"source_hash": h, "kernels": {}}
    prof.pop("summary", None)
    prof["kernels"][a.key] = {"summary": a.summary, "traffic_bytes_per_launch": round(per_f + per_w), "fetch_bytes_per_launch": round(per_f),
                              "write_bytes_per_launch": round(per_w), "gemm_calls": round(gemms),
                              "fetch_scale": round(fscale, 4), "write_scale": round(wscale, 4)}
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(prof, f, indent=1, sort_keys=True)
        f.write("\n")
    print(f"\nwritten under `{a.key}` to profiles/traffic_counters.json (source hash {h})")


def cmd_sq(a):
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in _counter_rows(a.dir):
        if a.kernel in r["Kernel_Name"]:
            acc[(_short(r["Kernel_Name"]), int(r["Grid_Size"]))][r["Counter_Name"]].append(float(r["Counter_Value"]))
    counters = sorted({c for g in acc.values() for c in g})
    print("| kernel | grid (threads) | dispatches | " + " | ".join(counters) + " |")
    print("|---|---|---|" + "---|" * len(counters))
    for (name, grid), g in sorted(acc.items()):
        n = max(len(v) for v in g.values())
        print(f"| `{name}` | {grid} | {n} | " + " | ".join(f"{statistics.mean(g[c]):.4g}" if g[c] else "" for c in counters) + " |")


def cmd_stats(a):
    print("| kernel | calls | total ms | average us | min us | max us | % of GPU time |")
    print("|---|---|---|---|---|---|---|")
    with open(_one(a.dir, "kernel_stats.csv")) as f:
        for r in csv.DictReader(f):
            if "w4a8::" in r["Name"]:
                print(f"| `{_short(r['Name'])}` | {r['Calls']} | {float(r['TotalDurationNs']) / 1e6:.2f} | "
                      f"{float(r['AverageNs']) / 1e3:.2f} | {float(r['MinNs']) / 1e3:.2f} | {float(r['MaxNs']) / 1e3:.2f} | "
                      f"{float(r['Percentage']):.2f} |")
    dur = collections.defaultdict(list)
    with open(_one(a.dir, "kernel_trace.csv")) as f:
        for r in csv.DictReader(f):
            if "w4a8::" in r["Kernel_Name"]:
                grid = int(r["Grid_Size_X"]) * int(r.get("Grid_Size_Y", 1) or 1)
                dur[(_short(r["Kernel_Name"]), grid)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    print("\n| kernel | grid (threads) | launches | median us | min us |")
    print("|---|---|---|---|---|")
    for (name, grid), v in sorted(dur.items()):
        print(f"| `{name}` | {grid} | {len(v)} | {statistics.median(v):.2f} | {min(v):.2f} |")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("traffic")
    t.add_argument("--fetch", required=True)
    t.add_argument("--write", required=True)
    t.add_argument("--kernel", required=True)
    t.add_argument("--key", required=True)
    t.add_argument("--calls-per-dispatch", type=float, default=1.0, help="GEMM calls per dispatch of the kernel")
    t.add_argument("--by-grid", action="store_true",
                   help="mean over grid sizes of the mean per dispatch (one GEMM shape per grid size, equal weights)")
    t.add_argument("--summary", default="profiles/")
    s = sub.add_parser("sq")
    s.add_argument("--dir", required=True)
    s.add_argument("--kernel", required=True)
    k = sub.add_parser("stats")
    k.add_argument("--dir", required=True)
    a = ap.parse_args()
    {"traffic": cmd_traffic, "sq": cmd_sq, "stats": cmd_stats}[a.cmd](a)


if __name__ == "__main__":
    main()
