"""Condense a rocprofv3 `--kernel-trace --stats --output-format csv` run into a short text table.

    python -m paper_2003_06795_amd.tune.prof_summary gpurun_out/prof_x/x_kernel_stats.csv [top]
"""
import csv
import sys


def main(path, top=12):
    rows = list(csv.DictReader(open(path)))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    print("%-100s %8s %12s %10s %6s" % ("kernel", "calls", "total_ms", "avg_us", "%"))
    for r in rows[:top]:
        name = r["Name"].replace("void ks::", "").replace("(ks::GemmParams)", "")
        print("%-100s %8d %12.3f %10.3f %6.2f" % (name[:100], int(r["Calls"]), float(r["TotalDurationNs"]) / 1e6,
                                                 float(r["AverageNs"]) / 1e3, float(r["Percentage"])))
    print("total kernel time %.3f ms over %d kernel symbols" % (total / 1e6, len(rows)))


if __name__ == "__main__":
    main(sys.argv[1], int(sys.argv[2]) if len(sys.argv) > 2 else 12)
