"""Score the DEPLOYED selector (ks_select of the built library) on a timing table, per
configuration: geometric mean of selected / exhaustive-best (paper Table I's score), the score
achievable inside the set of kernels the tree can return (Section III-A), and the best single
kernel.  Scores are computed by the library's host tuner.

    python -m paper_2003_06795_amd.tune.evaluate --dtype f32 --timings <csv> [--out report.json]
"""
import argparse
import json
import sys

import numpy as np

from .. import binding as ks
from . import train


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--timings", required=True)
    ap.add_argument("--out", default=None)
    a = ap.parse_args(argv)
    dt = ks.F32 if a.dtype == "f32" else ks.BF16
    rows, T = train.load_table(a.timings, a.dtype)
    P = train.perf_of(rows, T)
    Ph = ks.tune_normalise(P)
    chosen = np.array([ks.select(dt, r["M"], r["N"], r["K"], r["batch"], r["tA"], r["tB"]) for r in rows])
    leaves = sorted({int(n["value"]) for n in ks.get_selector(dt) if n["feature"] < 0})
    report = dict(dtype=a.dtype, timings=a.timings, tree_leaf_kernels=leaves, configs=[])
    for cfg in sorted({r["config"] for r in rows}):
        m = np.array([r["config"] == cfg for r in rows])
        report["configs"].append(dict(
            config=cfg, rows=int(m.sum()),
            selected_over_best_geomean=ks.tune_selector_score(Ph[m], chosen[m]),
            achievable_geomean=ks.tune_achievable(Ph[m], leaves),
            best_single_kernel_geomean=max(ks.tune_achievable(Ph[m], [c]) for c in range(P.shape[1])),
            best_tflops_geomean=float(np.exp(np.mean(np.log(P[m].max(axis=1) / 1e12)))),
            selected_tflops_geomean=float(np.exp(np.mean(np.log(P[m][np.arange(m.sum()), chosen[m]] / 1e12))))))
    text = json.dumps(report, indent=1)
    print(text)
    if a.out:
        open(a.out, "w").write(text + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
