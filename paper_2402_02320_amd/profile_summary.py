"""Condenses rocprofv3 CSV output (kernel stats or one counter pass) into the
few lines kept under profiles/.

    python -m paper_2402_02320_amd.profile_summary stats  <dir>   # --kernel-trace --stats --output-format csv
    python -m paper_2402_02320_amd.profile_summary pmc    <dir>   # --pmc ... --output-format csv
"""
import collections
import csv
import glob
import os
import sys


def _find(directory, suffix):
    hits = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit("no *%s under %s" % (suffix, directory))
    return hits[0]


def short(name):
    name = name.replace("spin::(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0][:70]


def stats(directory):
    rows = list(csv.DictReader(open(_find(directory, "kernel_stats.csv"))))
    print("%-72s %6s %12s %12s %7s" % ("kernel", "calls", "total_us", "avg_us", "pct"))
    for r in rows:
        if float(r["Percentage"]) < 0.05:
            continue
        print("%-72s %6d %12.1f %12.2f %7.2f" % (short(r["Name"]), int(r["Calls"]), float(r["TotalDurationNs"]) / 1e3,
                                                 float(r["AverageNs"]) / 1e3, float(r["Percentage"])))


def pmc(directory):
    rows = list(csv.DictReader(open(_find(directory, "counter_collection.csv"))))
    agg = collections.OrderedDict()
    for r in rows:
        key = (short(r["Kernel_Name"]), r["Counter_Name"])
        agg.setdefault(key, []).append(float(r["Counter_Value"]))
    print("%-72s %-28s %6s %16s %16s" % ("kernel", "counter", "calls", "mean", "max"))
    for (k, c), v in agg.items():
        if "at::native" in k or "at_cuda" in k:
            continue
        print("%-72s %-28s %6d %16.6g %16.6g" % (k, c, len(v), sum(v) / len(v), max(v)))


if __name__ == "__main__":
    if len(sys.argv) != 3 or sys.argv[1] not in ("stats", "pmc"):
        raise SystemExit(__doc__)
    {"stats": stats, "pmc": pmc}[sys.argv[1]](sys.argv[2])
