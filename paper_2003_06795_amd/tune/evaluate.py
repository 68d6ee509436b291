"""Score the DEPLOYED selector (ks_select of the built library) on a timing table, per
configuration: geometric mean of selected / exhaustive-best (paper Table I's score), the score
achievable inside the set of kernels the tree can return (Section III-A), and the best single
kernel.  Scores are computed by the library's host tuner.  Each row is also set against its
roofline bound min(matrix peak, arithmetic intensity x 8 TB/s) with the algorithmic bytes of the
call (operands once, C written once and read once when beta != 0): fraction reached by the best
and by the selected kernel.

    python -m paper_2003_06795_amd.tune.evaluate --dtype f32 --timings <csv> [--out report.json]
"""
import argparse
import json
import sys

import numpy as np

from .. import binding as ks
from . import train


PEAK_TFLOPS = {"f32": 157.3, "bf16": 2516.6}     # dense matrix-core peaks of MI355X
HBM_TBS = 8.0


def attainable(dtype, r, beta):
    """Roofline bound of one row in flop/s."""
    esz = 4 if dtype == "f32" else 2
    M, N, K, b = r["M"], r["N"], r["K"], r["batch"]
    by = b * ((M * K + K * N) * esz + M * N * 4 * (2 if beta else 1))
    return min(PEAK_TFLOPS[dtype] * 1e12, 2.0 * M * N * K * b / by * HBM_TBS * 1e12)


def quartiles(f):
    q = np.quantile(f, [0.25, 0.5, 0.75])
    return dict(geomean=float(np.exp(np.mean(np.log(f)))), q25=float(q[0]), median=float(q[1]),
                q75=float(q[2]), max=float(np.max(f)))


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
    # config 4 is the only table measured with beta != 0 (sweep.rows_of)
    bound = np.array([attainable(a.dtype, r, r["config"] == 4) for r in rows])
    for cfg in sorted({r["config"] for r in rows}):
        m = np.array([r["config"] == cfg for r in rows])
        sel = P[m][np.arange(m.sum()), chosen[m]]
        report["configs"].append(dict(
            config=cfg, rows=int(m.sum()),
            selected_over_best_geomean=ks.tune_selector_score(Ph[m], chosen[m]),
            achievable_geomean=ks.tune_achievable(Ph[m], leaves),
            best_single_kernel_geomean=max(ks.tune_achievable(Ph[m], [c]) for c in range(P.shape[1])),
            best_over_roofline_bound=quartiles(P[m].max(axis=1) / bound[m]),
            selected_over_roofline_bound=quartiles(sel / bound[m]),
            best_tflops_geomean=float(np.exp(np.mean(np.log(P[m].max(axis=1) / 1e12)))),
            selected_tflops_geomean=float(np.exp(np.mean(np.log(P[m][np.arange(m.sum()), chosen[m]] / 1e12))))))
    text = json.dumps(report, indent=1)
    print(text)
    if a.out:
        open(a.out, "w").write(text + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
