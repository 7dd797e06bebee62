"""Condense rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2605_15422_amd.profile_summary kernel-trace <dir>   # per (kernel, grid) durations
  python -m paper_2605_15422_amd.profile_summary pmc <dir>            # per (kernel, grid) counter averages
"""
import collections
import csv
import glob
import sys


def _name(r):
    return r["Kernel_Name"].replace("(anonymous namespace)::", "").split("(")[0].replace("void ", "")


def kernel_trace(d):
    f = glob.glob(d + "/**/*kernel_trace.csv", recursive=True)[0]
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(f)):
        k = "%s grid=%s block=%s" % (_name(r), r["Grid_Size_X"], r["Workgroup_Size_X"])
        agg[k].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    print("%-64s %5s %12s %12s %12s" % ("kernel", "calls", "avg_us", "min_us", "max_us"))
    for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
        print("%-64s %5d %12.1f %12.1f %12.1f" % (k, len(v), sum(v) / len(v), min(v), max(v)))


def pmc(d):
    f = glob.glob(d + "/**/*counter_collection.csv", recursive=True)[0]
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(f)):
        k = "%s grid=%s" % (_name(r), r["Grid_Size"])
        agg[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
    for k, cs in sorted(agg.items()):
        for c, v in sorted(cs.items()):
            print("%-64s %-28s calls=%d avg=%.6g" % (k, c, len(v), sum(v) / len(v)))


if __name__ == "__main__":
    {"kernel-trace": kernel_trace, "pmc": pmc}[sys.argv[1]](sys.argv[2])
