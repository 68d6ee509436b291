"""Condense a rocprofv3 `--kernel-trace --stats --output-format csv` run into a short text table.

    python -m paper_2003_06795_amd.tune.prof_summary <dir>/<name>_kernel_stats.csv [--bench <bench line .json>]
                                                     [--share 0.9] [--max-rows 60]

Prints the kernel symbols by total time until `share` of the kernel time is covered.  With --bench
(the JSON line bench.py printed in the profiled run) the row of the line's roofline kernel is
always printed, marked, with the TFLOP/s that follows from its average duration and the line's
flops per launch, so that the line's `roofline.frac` can be recomputed from this file alone; the
second kernel of the balanced persistent form (which shares the timed interval of its GEMM in the
bench line) is always printed too.
"""
import argparse
import csv
import json


def short(name):
    return name.replace("void ks::", "").replace("(ks::GemmParams)", "")


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("stats_csv")
    ap.add_argument("--bench", default=None)
    ap.add_argument("--share", type=float, default=0.9)
    ap.add_argument("--max-rows", type=int, default=60)
    a = ap.parse_args(argv)
    # the library's kernels only (the benchmark's data generation runs torch kernels)
    rows = [r for r in csv.DictReader(open(a.stats_csv)) if "ks::" in r["Name"]]
    rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    roof = None
    if a.bench:
        line = [l for l in open(a.bench) if l.startswith("{")][-1]
        roof = json.loads(line)["roofline"]
    print("%-100s %8s %12s %10s %6s" % ("kernel", "calls", "total_ms", "avg_us", "%"))
    cum, shown = 0.0, 0
    for r in rows:
        name = short(r["Name"])
        is_roof = roof is not None and name.startswith(roof["kernel"].rstrip(">"))
        if (cum < a.share * total and shown < a.max_rows) or is_roof or "sk_fixup" in name:
            print("%-100s %8d %12.3f %10.3f %6.2f%s" % (name[:100], int(r["Calls"]), float(r["TotalDurationNs"]) / 1e6,
                                                       float(r["AverageNs"]) / 1e3,
                                                       100.0 * float(r["TotalDurationNs"]) / total,
                                                       "  <- roofline kernel" if is_roof else ""))
            shown += 1
            if is_roof:
                tf = roof["flops_per_launch"] / (float(r["AverageNs"]) * 1e-9) / 1e12
                print("    roofline kernel from this file: %.4g flops per launch / %.3f us = %.2f TFLOP/s = %.3f of %.1f "
                      "(bench line: %.2f TFLOP/s, frac %.3f, avg %.3f us)" % (
                          roof["flops_per_launch"], float(r["AverageNs"]) / 1e3, tf, tf / roof["peak"], roof["peak"],
                          roof["achieved"], roof["frac"], roof["avg_launch_us"]))
        cum += float(r["TotalDurationNs"])
    print("total time of the library's kernels %.3f ms over %d symbols; the rows shown cover at least %.0f %% of it" % (
        total / 1e6, len(rows), 100.0 * (1.0 if shown == len(rows) else a.share)))


if __name__ == "__main__":
    main()
