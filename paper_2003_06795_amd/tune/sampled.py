"""Two-stage (sampled) tuning for configuration spaces too large to brute-force.

The paper's conclusion leaves open how to tune when timing every configuration on every workload
is too expensive.  This driver does the obvious thing with the pipeline of Sections III and IV:

  stage 1  time EVERY configuration on a seeded fraction of the training shapes only, normalise,
           and let the decision-tree pruner choose the kept set from those rows;
  stage 2  time only the KEPT configurations on the remaining training shapes, label every
           training row inside the kept set and fit the selector on all of them.

Cost: |stage 1 rows| x |family| + |other rows| x |kept| timed cells instead of |rows| x |family|.
Run on a stored exhaustive table, it reads only the cells the procedure would have timed and
reports what the shortcut costs against the full pipeline on the held-out shapes:

    python -m paper_2003_06795_amd.tune.sampled --dtype f32 --timings tune/data/timings_f32_cfg2.csv

For a live run, `sweep.py --kernels` times a chosen subset of kernel ids.
"""
import argparse
import json
import sys

import numpy as np

from .. import binding as ks
from . import train


def shape_key(r):
    return (r["config"], r["M"], r["N"], r["K"], r["batch"])


def stage1_mask(rows, fraction, seed):
    """Boolean mask over `rows`: all layouts of a seeded `fraction` of the distinct shapes."""
    shapes = sorted({shape_key(r) for r in rows})
    perm = np.random.default_rng([int(seed), 0x5A3D]).permutation(len(shapes))
    n = max(1, int(np.ceil(fraction * len(shapes))))
    chosen = {shapes[int(j)] for j in perm[:n]}
    return np.array([shape_key(r) in chosen for r in rows], dtype=bool)


def sampled_fit(X, P, mask, n_kept, max_depth=12, min_samples_leaf=1):
    """Library-side two-stage fit.  Returns kept ids, selector tree, timed cells."""
    kept, _ = ks.tune_prune_tree(X[mask], ks.tune_normalise(P[mask]), n_kept)
    measured = np.zeros_like(P)
    measured[:, kept] = P[:, kept]                  # nothing else is read from here on
    tree = ks.tune_fit_selector(X, measured, kept, max_depth=max_depth, min_samples_leaf=min_samples_leaf)
    cells = int(mask.sum()) * P.shape[1] + int((~mask).sum()) * len(kept)
    return kept, tree, cells


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--timings", required=True, nargs="+")
    ap.add_argument("--n-kept", type=int, default=15)
    ap.add_argument("--features", type=int, default=ks.NUM_FEATURES)
    ap.add_argument("--min-samples-leaf", type=int, default=1)
    ap.add_argument("--fractions", type=float, nargs="+", default=[0.05, 0.1, 0.2, 0.3, 0.5, 1.0])
    ap.add_argument("--seeds", type=int, default=5)
    ap.add_argument("--out", default=None)
    a = ap.parse_args(argv)
    rows, T = [], []
    for path in a.timings:
        r_, t_ = train.load_table(path, a.dtype)
        rows += r_
        T.append(t_)
    P = train.perf_of(rows, np.concatenate(T, axis=0))
    X = train.features_of(rows, a.features)
    tr, te = train.split_rows(rows)
    rows_tr = [r for r, m in zip(rows, tr) if m]
    Xtr, Ptr, Xte, Ph_te = X[tr], P[tr], X[te], ks.tune_normalise(P[te])
    full_cells = Ptr.shape[0] * Ptr.shape[1]
    report = dict(dtype=a.dtype, timings=a.timings, n_kept=a.n_kept, train_rows=int(tr.sum()),
                  test_rows=int(te.sum()), family=int(P.shape[1]), results=[])
    print("%8s %10s %8s %12s %10s   (mean over %d stage-1 draws; held-out rows)"
          % ("fraction", "cells", "kernels", "achievable", "selector", a.seeds))
    for f in a.fractions:
        acc = []
        for seed in range(a.seeds if f < 1.0 else 1):
            mask = stage1_mask(rows_tr, f, seed)
            kept, tree, cells = sampled_fit(Xtr, Ptr, mask, a.n_kept, min_samples_leaf=a.min_samples_leaf)
            acc.append((cells / full_cells, len(kept), ks.tune_achievable(Ph_te, kept),
                        ks.tune_selector_score(Ph_te, ks.tune_predict(tree, Xte))))
        m = np.mean(np.array(acc), axis=0)
        report["results"].append(dict(fraction=f, cells_ratio=float(m[0]), kernels=float(m[1]),
                                      achievable=float(m[2]), selector=float(m[3])))
        print("%8.2f %9.1f%% %8.1f %12.4f %10.4f" % (f, 100 * m[0], m[1], m[2], m[3]))
    if a.out:
        with open(a.out, "w") as fh:
            json.dump(report, fh, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
