"""Condense one rocprofv3 `--pmc <SQ counters> --output-format csv` run of bench.py into one line per
(kernel symbol, grid size): the counters summed over that cell's dispatches and the derived
fractions
    mfma_busy_frac = SQ_VALU_MFMA_BUSY_CYCLES / (4 * SQ_BUSY_CU_CYCLES)   (busy cycles are counted per
                     SIMD, four to a compute unit)
    wait_frac      = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES

    python -m paper_2003_06795_amd.tune.counter_summary <dir>/p_counter_collection.csv [min_share]

Only the library's kernels are listed.  Cells whose SQ_BUSY_CU_CYCLES is below `min_share` (default 0.01) of the run's total are left out.
"""
import collections
import csv
import re
import sys


def short(name):
    return re.sub(r"^void ks::|\(ks::GemmParams\)$", "", name)


def main(path, min_share=0.01):
    cells = collections.defaultdict(lambda: collections.defaultdict(float))
    launches = collections.Counter()
    seen = set()
    for r in csv.DictReader(open(path)):
        if "ks::" not in r["Kernel_Name"]:
            continue                          # the benchmark's data generation (torch kernels)
        key = (short(r["Kernel_Name"]), int(r["Grid_Size"]))
        cells[key][r["Counter_Name"]] += float(r["Counter_Value"])
        d = (r["Dispatch_Id"], key)
        if d not in seen:
            seen.add(d)
            launches[key] += 1
    total = sum(c.get("SQ_BUSY_CU_CYCLES", 0.0) for c in cells.values()) or 1.0
    for key in sorted(cells, key=lambda k: -cells[k].get("SQ_BUSY_CU_CYCLES", 0.0)):
        c = cells[key]
        if c.get("SQ_BUSY_CU_CYCLES", 0.0) < min_share * total:
            continue
        parts = ["%s=%.4g" % (n, c[n]) for n in sorted(c)]
        if c.get("SQ_BUSY_CU_CYCLES") and "SQ_VALU_MFMA_BUSY_CYCLES" in c:
            parts.append("mfma_busy_frac=%.3f" % (c["SQ_VALU_MFMA_BUSY_CYCLES"] / (4.0 * c["SQ_BUSY_CU_CYCLES"])))
        if c.get("SQ_WAVE_CYCLES") and "SQ_WAIT_INST_ANY" in c:
            parts.append("wait_frac=%.3f" % (c["SQ_WAIT_INST_ANY"] / c["SQ_WAVE_CYCLES"]))
        print("%s grid=%d launches=%d: %s" % (key[0], key[1], launches[key], ", ".join(parts)))


if __name__ == "__main__":
    main(sys.argv[1], float(sys.argv[2]) if len(sys.argv) > 2 else 0.01)
