"""Turn two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch) into
HBM bytes per launch for every GEMM kernel symbol, scaled by the calibration copy.

    python -m paper_2003_06795_amd.tune.pmc_summary FETCH.csv WRITE.csv cfg2 > profiles/pmc_traffic_cfg2.txt

Scaling: bench.py launches ks::copy_kernel once over a known number of bytes (read once, written
once).  factor = known KiB / counter KiB for that dispatch, separately for reads and writes, and
every other dispatch's counter is multiplied by it.
"""
import collections
import csv
import json
import re
import sys

CALIB_BYTES = 256 * 1024 * 1024


def per_kernel(path, counter):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            agg[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return agg


def short(name):
    return re.sub(r"^void ks::|\(ks::GemmParams\)$", "", name)


def main(fetch_csv, write_csv, workload):
    f, w = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    ck = [k for k in f if "copy_kernel" in k][0]
    ff = (CALIB_BYTES / 1024.0) / (sum(f[ck]) / len(f[ck]))
    wf = (CALIB_BYTES / 1024.0) / (sum(w[ck]) / len(w[ck]))
    out = dict(workload=workload,
               command=("rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir> -o p -- python3 bench.py "
                        "--workload %s --steps 1 --warmup 0 --no-cpu --no-extra --single-launch  (and the same with "
                        "--pmc WRITE_SIZE); python -m paper_2003_06795_amd.tune.pmc_summary "
                        "<fetch>/p_counter_collection.csv <write>/p_counter_collection.csv %s" % (workload, workload)),
               calibration=dict(kernel=short(ck), bytes_each_way=CALIB_BYTES,
                                                   fetch_factor=ff, write_factor=wf), kernels=[])
    for k in sorted(f):
        if "gemm_" not in k:
            continue
        out["kernels"].append(dict(kernel=short(k), launches=len(f[k]),
                                   fetch_bytes=ff * 1024.0 * sum(f[k]) / len(f[k]),
                                   write_bytes=wf * 1024.0 * sum(w.get(k, [0])) / max(len(w.get(k, [0])), 1)))
    print(json.dumps(out, indent=1))


if __name__ == "__main__":
    main(*sys.argv[1:4])
