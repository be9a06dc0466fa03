"""Condenses rocprofv3 output folders into the short tables kept under profiles/.

    python3 -m paper_2410_03348_amd.profile_summary stats <dir>      # of a --kernel-trace --stats run
    python3 -m paper_2410_03348_amd.profile_summary pmc <dir> [...]  # of --pmc runs (one counter each)

`stats` prints calls / total / average / min / max per kernel; `pmc` prints the per-dispatch average of every
counter per kernel (FETCH_SIZE and WRITE_SIZE are in KiB).  Only kernels of this library and the runtime's copy
kernel are listed unless --all is given.
"""
import argparse
import collections
import csv
import glob
import os


def _short(name):
    name = name.split("(")[0].strip()
    return name[5:] if name.startswith("void ") else name


def _ours(name):
    return "dol::" in name or "copyBuffer" in name or name.startswith(("damp_", "dtkp_", "void damp_", "void dtkp_"))


def stats(folder, everything=False):
    rows = []
    for f in glob.glob(os.path.join(folder, "**", "*kernel_stats.csv"), recursive=True):
        for r in csv.DictReader(open(f)):
            if everything or _ours(r["Name"]):
                rows.append((_short(r["Name"]), int(r["Calls"]), float(r["TotalDurationNs"]) / 1e6,
                             float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3))
    rows.sort(key=lambda r: -r[2])
    print("| kernel | calls | total ms | avg us | min us | max us |")
    print("|---|---|---|---|---|---|")
    for r in rows:
        print("| `%s` | %d | %.3f | %.2f | %.2f | %.2f |" % r)


def pmc(folders, everything=False):
    agg = collections.defaultdict(lambda: collections.defaultdict(lambda: [0.0, 0]))
    for folder in folders:
        for f in glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                if everything or _ours(r["Kernel_Name"]):
                    a = agg[_short(r["Kernel_Name"])][r["Counter_Name"]]
                    a[0] += float(r["Counter_Value"])
                    a[1] += 1
    counters = sorted({c for k in agg.values() for c in k})
    print("| kernel | dispatches | " + " | ".join("%s / dispatch" % c for c in counters) + " |")
    print("|---|---|" + "---|" * len(counters))
    for k in sorted(agg):
        n = max(v[1] for v in agg[k].values())
        cells = ["%.1f" % (agg[k][c][0] / agg[k][c][1]) if c in agg[k] else "-" for c in counters]
        print("| `%s` | %d | %s |" % (k, n, " | ".join(cells)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["stats", "pmc"])
    ap.add_argument("folders", nargs="+")
    ap.add_argument("--all", action="store_true")
    args = ap.parse_args()
    if args.what == "stats":
        for f in args.folders:
            stats(f, args.all)
    else:
        pmc(args.folders, args.all)


if __name__ == "__main__":
    main()
