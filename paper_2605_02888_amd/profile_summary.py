"""Condense rocprofv3 CSV output to the few lines that concern this library's kernels.

    python -m paper_2605_02888_amd.profile_summary <rocprofv3 output dir> [more dirs ...]

For every *_kernel_stats.csv found: calls, average / min / max duration of each speckv kernel.
For every *_counter_collection.csv found: the mean counter value per dispatch of each speckv
kernel (FETCH_SIZE and WRITE_SIZE are reported by the profiler in KiB per dispatch).
"""
import collections
import csv
import os
import re
import sys


def short(name: str) -> str:
    name = re.sub(r"^void ", "", name)
    name = re.sub(r"\(.*$", "", name)
    return name.replace("speckv::", "")


def find(root, suffix):
    for dirpath, _, files in os.walk(root):
        for f in sorted(files):
            if f.endswith(suffix):
                yield os.path.join(dirpath, f)


def kernel_stats(path):
    print(f"# {os.path.basename(path)}")
    print(f"{'kernel':<58}{'calls':>7}{'avg_us':>10}{'min_us':>10}{'max_us':>10}{'total_ms':>10}")
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            if "speckv" not in row["Name"]:
                continue
            print(f"{short(row['Name']):<58}{int(row['Calls']):>7}{float(row['AverageNs']) / 1e3:>10.2f}"
                  f"{float(row['MinNs']) / 1e3:>10.2f}{float(row['MaxNs']) / 1e3:>10.2f}"
                  f"{float(row['TotalDurationNs']) / 1e6:>10.3f}")


def counters(path):
    acc = collections.defaultdict(list)
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            if "speckv" not in row["Kernel_Name"]:
                continue
            acc[(short(row["Kernel_Name"]), row["Counter_Name"])].append(float(row["Counter_Value"]))
    print(f"# {os.path.basename(path)}")
    print(f"{'kernel':<58}{'counter':>12}{'dispatches':>11}{'mean':>16}{'min':>16}{'max':>16}")
    for (k, c), v in sorted(acc.items()):
        print(f"{k:<58}{c:>12}{len(v):>11}{sum(v) / len(v):>16.1f}{min(v):>16.1f}{max(v):>16.1f}")


def main(argv):
    if not argv:
        print(__doc__)
        return 2
    for root in argv:
        for p in find(root, "_kernel_stats.csv"):
            kernel_stats(p)
        for p in find(root, "_counter_collection.csv"):
            counters(p)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
