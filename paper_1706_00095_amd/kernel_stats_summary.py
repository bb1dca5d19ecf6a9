#!/usr/bin/env python3
"""Text summary of a rocprofv3 --kernel-trace --stats run of bench.py (the library's kernels only).

    python3 paper_1706_00095_amd/kernel_stats_summary.py <dir>/<prefix>_kernel_stats.csv <out.txt> "<title>" "<command>"
"""
import csv
import re
import sys


def main():
    src, out, title, cmd = sys.argv[1:5]
    rows = [r for r in csv.DictReader(open(src)) if "cg::" in r["Name"]]
    total = sum(int(r["TotalDurationNs"]) for r in rows)
    with open(out, "w") as f:
        f.write(f"# {title}\n# command (from the repository root on the MI355X box):\n#   {cmd}\n")
        f.write("# source: rocprofv3's <prefix>_kernel_stats.csv; the library's kernels only (torch's fill / random-number\n")
        f.write("# kernels of the input set-up omitted); % is of the listed kernels' total time\n")
        f.write(f"{'kernel':96s} {'calls':>6s} {'total_ms':>10s} {'avg_us':>10s} {'min_us':>9s} {'max_us':>9s} {'%':>6s}\n")
        for r in rows:
            n = re.sub(r"\(anonymous namespace\)::", "", r["Name"])
            n = re.sub(r"\(.*$", "", n).replace("void ", "")
            f.write(f"{n[:96]:96s} {int(r['Calls']):6d} {int(r['TotalDurationNs']) / 1e6:10.3f} "
                    f"{float(r['AverageNs']) / 1e3:10.2f} {int(r['MinNs']) / 1e3:9.2f} {int(r['MaxNs']) / 1e3:9.2f} "
                    f"{100.0 * int(r['TotalDurationNs']) / total:6.2f}\n")


if __name__ == "__main__":
    main()
