"""Matrix-pipeline occupancy per kernel from one rocprofv3 counter run.

    rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES --kernel-trace --output-format csv \\
              -d <dir> -o m -- python3 bench.py <bench arguments>
    python3 paper_1706_00095_amd/pmc_mfma_busy.py <dir>/m_counter_collection.csv \\
              <dir>/m_kernel_trace.csv <out.txt> '<bench arguments>'

Per kernel label (the labels of pmc_traffic.py), over the matrix-core launches of the run:
  busy    = SQ_BUSY_CU_CYCLES / (duration x 2.4 GHz x 256 compute units): share of the launch's duration in
            which a compute unit has a wave (the rest: rounds of blocks that do not fill the chip, start-up);
  mfma    = SQ_VALU_MFMA_BUSY_CYCLES / (4 x SQ_BUSY_CU_CYCLES): share of that time in which the matrix
            pipeline of a SIMD is executing;
  product = mfma busy over the whole duration, to compare with the launch's TFLOP/s over the 157.3 peak.
"""
import collections
import csv
import sys

from pmc_traffic import label

CLOCK_GHZ, CUS, SIMDS = 2.4, 256, 4


def main():
    counters, trace, out, args = sys.argv[1:5]
    dur = {r["Dispatch_Id"]: int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) for r in csv.DictReader(open(trace))}
    per = collections.defaultdict(dict)
    name = {}
    for r in csv.DictReader(open(counters)):
        if "cg::igemm" not in r["Kernel_Name"]:
            continue
        per[r["Dispatch_Id"]][r["Counter_Name"]] = float(r["Counter_Value"])
        name[r["Dispatch_Id"]] = label(r["Kernel_Name"])
    agg = collections.defaultdict(lambda: [0, 0.0, 0.0, 0.0])
    for did, c in per.items():
        if "SQ_BUSY_CU_CYCLES" not in c or "SQ_VALU_MFMA_BUSY_CYCLES" not in c or did not in dur:
            continue
        a = agg[name[did]]
        a[0] += 1; a[1] += dur[did]; a[2] += c["SQ_BUSY_CU_CYCLES"]; a[3] += c["SQ_VALU_MFMA_BUSY_CYCLES"]
    with open(out, "w") as f:
        f.write("# Matrix-pipeline occupancy of the matrix-core kernels (hardware counters, one run)\n")
        f.write("# command (from the repository root on the MI355X box):\n")
        f.write("#   rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES --kernel-trace --output-format csv "
                f"-d gpurun_out/pmc_m -o m -- python3 bench.py {args}\n")
        f.write("#   python3 paper_1706_00095_amd/pmc_mfma_busy.py <counter csv> <kernel trace csv> <this file> '<args>'\n")
        f.write("# busy = compute units with work / duration; mfma = matrix pipeline executing / busy; product = over the duration\n")
        f.write(f"{'kernel label':36s} {'launches':>8s} {'avg us':>9s} {'busy %':>7s} {'mfma %':>7s} {'product %':>9s}\n")
        for lab, (n, ns, busy, mfma) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
            cu_cycles = ns * CLOCK_GHZ * CUS
            f.write(f"{lab:36s} {n:8d} {ns / n / 1e3:9.1f} {100 * busy / cu_cycles:7.1f} {100 * mfma / (SIMDS * busy):7.1f} "
                    f"{100 * mfma / (SIMDS * cu_cycles):9.1f}\n")


if __name__ == "__main__":
    main()
