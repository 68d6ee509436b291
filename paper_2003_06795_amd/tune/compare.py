"""Reproduce the shape of the paper's Figure 3 (PCA variance), Figure 4 (pruning methods vs number
of kept kernels) and Table I (selector vs other classifiers) on a measured timing table.

    python -m paper_2003_06795_amd.tune.compare --dtype f32 --timings <csv> [--out report.json]

Pruning (top-N by wins, k-means, PCA + k-means, HDBSCAN, decision tree), the PCA spectrum, the selector
tree and every score are computed by the library's host tuner (ks_tune_*).  The other classifiers
of Table I are comparison systems, not part of the library: they are run with scikit-learn when it
is importable (as in the paper) and skipped otherwise.
"""
import argparse
import json
import sys

import numpy as np

from .. import binding as ks
from . import train


def other_classifiers(Xtr, ytr, Xte):
    try:
        from sklearn.ensemble import RandomForestClassifier
        from sklearn.neighbors import KNeighborsClassifier
        from sklearn.pipeline import make_pipeline
        from sklearn.preprocessing import StandardScaler
        from sklearn.svm import SVC, LinearSVC
    except Exception:
        return {}
    lx = lambda X: np.log2(np.maximum(X.astype(np.float64), 1.0))
    models = {
        "RandomForest": RandomForestClassifier(n_estimators=100, random_state=0),
        "1NearestNeighbor": make_pipeline(StandardScaler(), KNeighborsClassifier(1)),
        "3NearestNeighbors": make_pipeline(StandardScaler(), KNeighborsClassifier(3)),
        "LinearSVM": make_pipeline(StandardScaler(), LinearSVC(random_state=0, max_iter=20000)),
        "RadialSVM": make_pipeline(StandardScaler(), SVC(kernel="rbf", random_state=0)),
    }
    out = {}
    for name, m in models.items():
        if len(set(ytr.tolist())) < 2:
            out[name] = np.full(Xte.shape[0], ytr[0])
            continue
        m.fit(lx(Xtr), ytr)
        out[name] = m.predict(lx(Xte)).astype(np.int32)
    return out


def hdbscan_pruning(Ph_tr, Ph_te):
    """HDBSCAN has no "number of clusters" parameter: sweep its minimum cluster size (the library's
    ks_tune_prune_hdbscan, minimum samples = minimum cluster size) and report what each setting keeps."""
    out, seen = [], set()
    for mcs in (2, 3, 4, 5, 6, 8, 10, 15, 20, 30, 40):
        kept, labels = ks.tune_prune_hdbscan(Ph_tr, mcs)
        key = tuple(kept.tolist())
        if key in seen:
            continue
        seen.add(key)
        out.append(dict(min_cluster_size=mcs, clusters=int(labels.max()) + 1, noise_rows=int((labels < 0).sum()),
                        kept=kept.tolist(), achievable=ks.tune_achievable(Ph_te, kept)))
    return sorted(out, key=lambda r: len(r["kept"]))


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--timings", required=True, nargs="+")
    ap.add_argument("--features", type=int, default=ks.NUM_FEATURES)
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
    Ph_tr, Ph_te = ks.tune_normalise(P[tr]), ks.tune_normalise(P[te])

    ratio = ks.tune_pca_variance(Ph_tr)
    cum = np.cumsum(ratio)
    need = {str(f): int(np.searchsorted(cum, f - 1e-12) + 1) for f in (0.8, 0.9, 0.95)}
    dims = need["0.95"]
    wins = np.bincount(np.argmax(P, axis=1), minlength=P.shape[1])
    report = dict(dtype=a.dtype, timings=a.timings, rows=len(rows), train_rows=int(tr.sum()), test_rows=int(te.sum()),
                  win_counts=dict(top=int(wins.max()), runner_up=int(np.sort(wins)[-2]),
                                  distinct_winners=int((wins > 0).sum())),
                  worst_kernel_best_case=float(ks.tune_normalise(P).max(axis=0).min()),
                  pca=dict(variance_ratio=[float(v) for v in ratio[:16]], components_for=need),
                  pruning=[], classifiers=[])
    print("PCA: components for 80/90/95 %% of the variance: %s" % need)
    print("wins: top kernel %d rows, runner-up %d, %d distinct winners; the weakest kernel's best case is %.2f of optimal"
          % (report["win_counts"]["top"], report["win_counts"]["runner_up"], report["win_counts"]["distinct_winners"],
             report["worst_kernel_best_case"]))
    print("%3s %9s %9s %9s %9s   (held-out achievable score)" % ("N", "top-N", "k-means", "PCA+km", "tree"))
    for n in range(4, 16):
        kept = dict(top_n=ks.tune_prune_top_n(Ph_tr, n), kmeans=ks.tune_prune_kmeans(Ph_tr, n),
                    pca_kmeans=ks.tune_prune_kmeans(Ph_tr, n, pca_dims=dims),
                    tree=ks.tune_prune_tree(X[tr], Ph_tr, n)[0])
        row = dict(n=n)
        for k, v in kept.items():
            row[k] = dict(kept=v.tolist(), achievable=ks.tune_achievable(Ph_te, v))
        report["pruning"].append(row)
        print("%3d %9.4f %9.4f %9.4f %9.4f" % (n, row["top_n"]["achievable"], row["kmeans"]["achievable"],
                                               row["pca_kmeans"]["achievable"], row["tree"]["achievable"]))
    report["hdbscan"] = hdbscan_pruning(Ph_tr, Ph_te)
    for r in report["hdbscan"]:
        print("HDBSCAN min_cluster_size %2d: %2d clusters, %3d noise rows, %2d kernels kept, achievable %.4f"
              % (r["min_cluster_size"], r["clusters"], r["noise_rows"], len(r["kept"]), r["achievable"]))
    for n in (5, 6, 8, 15):
        kept = ks.tune_prune_tree(X[tr], Ph_tr, n)[0]
        tree = ks.tune_fit_selector(X[tr], P[tr], kept)
        row = dict(n=n, kept=kept.tolist(), achievable=ks.tune_achievable(Ph_te, kept),
                   DecisionTree=ks.tune_selector_score(Ph_te, ks.tune_predict(tree, X[te])))
        # labels for the comparison classifiers: the fastest kept kernel of each training row
        ytr = kept[np.argmax(P[tr][:, kept], axis=1)]
        for name, pred in other_classifiers(X[tr], ytr, X[te]).items():
            row[name] = ks.tune_selector_score(Ph_te, pred)
        report["classifiers"].append(row)
        print("N=%2d achievable %.4f | " % (n, row["achievable"]) +
              "  ".join("%s %.4f" % (k, v) for k, v in row.items() if k not in ("n", "kept", "achievable")))
    if a.out:
        with open(a.out, "w") as f:
            json.dump(report, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
