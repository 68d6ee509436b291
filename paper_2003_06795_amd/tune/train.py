"""Prune the kernel family and train the runtime selector from a timing table
(paper Sections II-A, III, III-A, IV), then emit the deployed tree.

    python -m paper_2003_06795_amd.tune.train --dtype f32 \
        --timings paper_2003_06795_amd/tune/data/timings_f32_cfg2.csv --n-kept 8 --emit

All arithmetic (normalisation, regression-tree pruning, scores, classifier fit, prediction) runs in
the library's host tuner (ks_tune_*); this file only loads the CSV, splits it and writes results.
Rows are split by SHAPE (the transposed variants of one shape stay together), 70/30, seeded.
"""
import argparse
import csv
import json
import os
import sys

import numpy as np

import workloads as wl
from .. import binding as ks

HERE = os.path.dirname(os.path.abspath(__file__))
DATA = os.path.join(HERE, "data")
TABLE_INC = os.path.join(os.path.dirname(HERE), "csrc", "selector_table.inc")


def load_table(path, dtype):
    """-> (rows: list of dict(row, tA, tB, M, N, K, batch), T: seconds [rows x kernels])"""
    nk = ks.num_kernels(ks.F32 if dtype == "f32" else ks.BF16)
    cells, meta = {}, {}
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["dtype"] != dtype:
                continue
            key = (int(r["config"]), int(r["row"]))
            meta[key] = dict(config=key[0], row=key[1], tA=int(r["transA"]), tB=int(r["transB"]),
                             M=int(r["M"]), N=int(r["N"]), K=int(r["K"]), batch=int(r["batch"]))
            cells.setdefault(key, {})[int(r["kernel"])] = float(r["median_ms"]) * 1e-3
    keys = sorted(k for k in cells if len(cells[k]) == nk)
    T = np.array([[cells[k][c] for c in range(nk)] for k in keys], dtype=np.float64)
    return [meta[k] for k in keys], T


def features_of(rows, n_features):
    return np.stack([ks.features(r["M"], r["N"], r["K"], r["batch"], r["tA"], r["tB"])[:n_features]
                     for r in rows])


def perf_of(rows, T):
    """Section II-A: flop/s of every configuration on every workload (computed by the library)."""
    return ks.tune_performance([[r["M"], r["N"], r["K"], r["batch"]] for r in rows], T)


def split_rows(rows):
    """Train/test masks by SHAPE, 70/30, seeded.  Config 2 (fp32 tuning set, 4 layouts per shape)
    and config 6 (bf16 tuning set, 2 layouts per shape) use the permutations defined with the
    workloads; configs 3 and 4 (one row per shape) are split by a permutation of the shapes present
    in the table seeded with the config number; the named bf16 large/skinny cells (config 5) are
    training rows only."""
    tr = np.zeros(len(rows), dtype=bool)
    te = np.zeros(len(rows), dtype=bool)
    s2, s6 = wl.config2_split(), wl.bf16_tuning_split()
    other = {}
    for cfg in (3, 4):
        ids = sorted({r["row"] for r in rows if r["config"] == cfg})
        perm = np.random.default_rng([cfg, 0x5917]).permutation(len(ids))
        n_train = int(round(0.7 * len(ids)))
        other[cfg] = {ids[int(j)] for j in perm[:n_train]}
    for i, r in enumerate(rows):
        if r["config"] == 2:
            tr[i], te[i] = r["row"] // 4 in s2[0], r["row"] // 4 in s2[1]
        elif r["config"] == 6:
            tr[i], te[i] = r["row"] // 2 in s6[0], r["row"] // 2 in s6[1]
        elif r["config"] in other:
            tr[i] = r["row"] in other[r["config"]]
            te[i] = not tr[i]
        elif r["config"] == 12:
            # large fp32 shapes: every other shape is held out
            tr[i], te[i] = (r["row"] // 4) % 2 == 0, (r["row"] // 4) % 2 == 1
        else:
            tr[i] = True
    return tr, te


LAYOUTS_PER_SHAPE = {2: 4, 7: 4, 12: 4, 13: 4, 6: 2, 8: 2, 5: 2}      # rows of one shape are consecutive in these configs


def validation_split(rows, tr, fraction=0.2, seed=0x5a17):
    """Carves a validation set out of the TRAINING rows, by shape (the layouts of a shape stay
    together), seeded: hyper-parameters (leaf limits, rows per classifier leaf) are chosen on it, so
    that the held-out test rows are looked at once, for the final number.  -> (fit mask, validation mask)"""
    groups = {}
    for i, r in enumerate(rows):
        if tr[i]:
            groups.setdefault((r["config"], r["row"] // LAYOUTS_PER_SHAPE.get(r["config"], 1)), []).append(i)
    keys = sorted(groups)
    perm = np.random.default_rng([seed, len(keys)]).permutation(len(keys))
    n_val = int(round(fraction * len(keys)))
    fit_m = np.zeros(len(rows), dtype=bool)
    val_m = np.zeros(len(rows), dtype=bool)
    for j, k in enumerate(perm):
        (val_m if j < n_val else fit_m)[groups[keys[int(k)]]] = True
    return fit_m, val_m


def fit(Xtr, Ptr, n_kept, max_depth, min_samples_leaf, weighted, prune=None):
    """prune: optional boolean mask of the rows the pruning tree sees (the classifier sees all)."""
    Ph = ks.tune_normalise(Ptr)
    if prune is None or prune.all():
        kept, reg = ks.tune_prune_tree(Xtr, Ph, n_kept)
    else:
        kept, reg = ks.tune_prune_tree(Xtr[prune], Ph[prune], n_kept)
    w = None
    if weighted:
        # optional, not in the paper: weight a row by what a wrong choice inside the kept set can
        # cost there (1 - worst/best normalised performance among kept configurations)
        sub = Ph[:, kept]
        w = 1.0 - sub.min(axis=1) / sub.max(axis=1) + 1e-3
    tree = ks.tune_fit_selector(Xtr, Ptr, kept, max_depth=max_depth,
                                min_samples_leaf=min_samples_leaf, row_weight=w)
    return kept, reg, tree


BATCH_FEATURE = 3          # index of `batch` in the ks_features layout


def fit_by_regime(Xtr, Ptr, n_single, n_batched, max_depth, min_samples_leaf, weighted, prune=None):
    """One pruning + classifier fit per regime (single GEMMs, batch == 1; batched ones, batch > 1),
    each with its own leaf limit, joined under a root that compares the batch count: the deployed
    selector stays one tree of nested comparisons (Section IV), but the rows of one regime no
    longer compete with the other's for the pruning tree's leaves (Section III)."""
    single = Xtr[:, BATCH_FEATURE] <= 1
    if prune is None:
        prune = np.ones(len(Xtr), dtype=bool)
    if single.all() or not single.any():
        return fit(Xtr, Ptr, n_single, max_depth, min_samples_leaf, weighted, prune)
    k1, r1, t1 = fit(Xtr[single], Ptr[single], n_single, max_depth, min_samples_leaf, weighted, prune[single])
    k2, r2, t2 = fit(Xtr[~single], Ptr[~single], n_batched, max_depth, min_samples_leaf, weighted, prune[~single])

    def join(a, b):
        out = np.zeros(1 + len(a) + len(b), dtype=ks.TREE_DTYPE)
        out[0] = (BATCH_FEATURE, 1, 1 + len(a), int(a[0]["value"]), 1)
        for off, part in ((1, a), (1 + len(a), b)):
            for i, n in enumerate(part):
                leaf = n["feature"] < 0
                out[off + i] = (n["feature"], -1 if leaf else n["left"] + off, -1 if leaf else n["right"] + off,
                                n["value"], n["threshold"])
        return out

    kept = np.array(sorted(set(k1.tolist()) | set(k2.tolist())), dtype=k1.dtype)
    return kept, join(r1, r2), join(t1, t2)


def evaluate(tree, kept, X, P, flops=None):
    """Scores of Section III-A / Table I on the rows given; with the rows' flop counts also the
    ratio of summed times, best kernels over selected kernels (the geometric mean weighs every row
    alike, the summed time is carried by the large ones)."""
    Ph = ks.tune_normalise(P)
    chosen = ks.tune_predict(tree, X)
    out = dict(achievable=ks.tune_achievable(Ph, kept), selector=ks.tune_selector_score(Ph, chosen),
               best_single=max(ks.tune_achievable(Ph, [c]) for c in range(P.shape[1])))
    if flops is not None:
        t = flops[:, None] / P
        out["time_ratio"] = float(t.min(axis=1).sum() / t[np.arange(len(t)), chosen].sum())
    return out


def emit_table(trees):
    """trees: {'f32': structured array, 'bf16': structured array} -> csrc/selector_table.inc"""
    lines = [
        "// Deployed decision trees (paper Section IV), one per operand type.",
        "// Written by paper_2003_06795_amd/tune/train.py from a measured timing table; do not edit.",
        "// {feature, left, right, value, threshold}: feature < 0 is a leaf choosing kernel `value`;",
        "// otherwise go left when features[feature] <= threshold.",
    ]
    for dtype, name in (("f32", "kTreeF32"), ("bf16", "kTreeBf16")):
        lines.append("static const ks_tree_node_t %s[] = {" % name)
        for n in trees[dtype]:
            lines.append("    {%d, %d, %d, %d, %dLL}," % (n["feature"], n["left"], n["right"], n["value"],
                                                          n["threshold"]))
        lines.append("};")
    with open(TABLE_INC, "w") as f:
        f.write("\n".join(lines) + "\n")


KEPT_INC = os.path.join(os.path.dirname(HERE), "csrc", "kept_set.inc")
BRING_UP_F32 = [0, 2, 4, 6]          # the four first-configuration tiles stay in every build


def emit_kept_set(trees):
    """csrc/kept_set.inc: the members a pruned build compiles = the leaves of the deployed trees
    (plus the four bring-up tiles)."""
    kept = {dt: sorted({int(n["value"]) for n in t if n["feature"] < 0}) for dt, t in trees.items()}
    # a kept member with a fixed split needs its twin without split: ks_gemm_* runs that one when no
    # workspace (or too small a one) is registered
    for dt, code in (("f32", ks.F32), ("bf16", ks.BF16)):
        infos = [ks.kernel_info(code, i) for i in range(ks.num_kernels(code))]
        same = lambda a, b: all(a[k] == b[k] for k in ("core", "bm", "bn", "wm", "wn", "tm", "tn", "k_waves"))
        for i in list(kept[dt]):
            if infos[i]["split_k"] > 1:
                twins = [j for j, e in enumerate(infos) if e["split_k"] == 1 and same(e, infos[i])]
                twins.sort(key=lambda j: (infos[j]["bk"] != infos[i]["bk"], j))
                if twins and twins[0] not in kept[dt]:
                    kept[dt].append(twins[0])
        kept[dt].sort()
    f32 = sorted(set(kept["f32"]) | set(BRING_UP_F32))
    lines = ["// Kernel ids a pruned build (-DKS_KEPT_ONLY) compiles: the leaves of the deployed trees and the",
             "// four bring-up tiles.  Written by paper_2003_06795_amd/tune/train.py with selector_table.inc; do not edit.",
             "#define KS_KEPT_F32 {" + ", ".join(str(i) for i in f32) + "}",
             "#define KS_KEPT_BF16 {" + ", ".join(str(i) for i in kept["bf16"]) + "}"]
    with open(KEPT_INC, "w") as f:
        f.write("\n".join(lines) + "\n")


def tree_to_json(tree):
    return [[int(n["feature"]), int(n["left"]), int(n["right"]), int(n["value"]), int(n["threshold"])]
            for n in tree]


def tree_from_json(rows):
    t = np.zeros(len(rows), dtype=ks.TREE_DTYPE)
    for i, r in enumerate(rows):
        t[i] = tuple(r)
    return t


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--timings", required=True, nargs="+", help="one or more timing tables (rows are pooled)")
    ap.add_argument("--n-kept", type=int, default=8)
    ap.add_argument("--max-depth", type=int, default=12)
    ap.add_argument("--min-samples-leaf", type=int, default=1)
    ap.add_argument("--features", type=int, default=ks.NUM_RAW_FEATURES,
                    help="length of the feature prefix (6 = raw sizes and flags, 10 = with derived)")
    ap.add_argument("--weighted", action="store_true")
    ap.add_argument("--n-kept-batched", type=int, default=0,
                    help="> 0: rows with batch > 1 are pruned and classified on their own with this leaf "
                         "limit, and the two trees are joined under a root that compares the batch count")
    ap.add_argument("--all-rows", action="store_true", help="train on every row (no held-out set)")
    ap.add_argument("--classifier-only-configs", default="",
                    help="comma list of config numbers whose training rows join the classifier fit but not the "
                         "pruning step (rows that would otherwise pull the few leaves of the pruning tree away)")
    ap.add_argument("--choose-by-validation", action="store_true",
                    help="choose --n-kept (among 4, 5, 6, 8, 12, 15), --n-kept-batched (4, 8; only if given > 0) and "
                         "--min-samples-leaf (1, 4, 8) on a validation split of the training shapes, then refit on "
                         "all training rows; the test rows are scored once, with the chosen setting")
    ap.add_argument("--emit", action="store_true", help="write tree JSON + csrc/selector_table.inc")
    ap.add_argument("--report", default=None)
    a = ap.parse_args(argv)

    rows, T = [], []
    for path in a.timings:
        r_, t_ = load_table(path, a.dtype)
        rows += r_
        T.append(t_)
    T = np.concatenate(T, axis=0)
    P = perf_of(rows, T)
    X = features_of(rows, a.features)
    F = np.array([2.0 * r["M"] * r["N"] * r["K"] * r["batch"] for r in rows])
    if a.all_rows:
        tr = te = np.ones(len(rows), dtype=bool)
    else:
        tr, te = split_rows(rows)
    conly = {int(c) for c in a.classifier_only_configs.split(",") if c}
    prune_rows = np.array([r["config"] not in conly for r in rows])
    if a.choose_by_validation:
        fit_m, val_m = validation_split(rows, tr)
        trials = []
        for n in (4, 5, 6, 8, 12, 15):
            for nb in ((4, 8) if a.n_kept_batched > 0 else (0,)):
                for msl in (1, 4, 8):
                    if nb > 0:
                        kept, _, tree = fit_by_regime(X[fit_m], P[fit_m], n, nb, a.max_depth, msl, a.weighted,
                                                      prune_rows[fit_m])
                    else:
                        kept, _, tree = fit(X[fit_m], P[fit_m], n, a.max_depth, msl, a.weighted, prune_rows[fit_m])
                    ev = evaluate(tree, kept, X[val_m], P[val_m], F[val_m])
                    trials.append(dict(n_kept=n, n_kept_batched=nb, min_samples_leaf=msl, kernels=len(kept),
                                       validation_selector=ev["selector"], validation_achievable=ev["achievable"]))
        # the fewest kernels among the settings within 0.002 of the best validation score (a smaller
        # library is what pruning is for); the better score on ties
        top = max(t["validation_selector"] for t in trials)
        best = min((t for t in trials if t["validation_selector"] >= top - 0.002),
                   key=lambda t: (t["kernels"], -t["validation_selector"]))
        print("chosen on %d validation rows (fit on %d): n_kept %d, n_kept_batched %d, min_samples_leaf %d "
              "(validation selector %.4f)" % (int(val_m.sum()), int(fit_m.sum()), best["n_kept"],
                                              best["n_kept_batched"], best["min_samples_leaf"],
                                              best["validation_selector"]))
        a.n_kept, a.n_kept_batched, a.min_samples_leaf = best["n_kept"], best["n_kept_batched"], best["min_samples_leaf"]
    report = dict(dtype=a.dtype, timings=[os.path.relpath(t) for t in a.timings], rows=len(rows),
                  train_rows=int(tr.sum()), test_rows=int(te.sum()), features=a.features,
                  max_depth=a.max_depth, min_samples_leaf=a.min_samples_leaf, weighted=a.weighted,
                  n_kept_batched=a.n_kept_batched, classifier_only_configs=sorted(conly), sweep=[])
    if a.choose_by_validation:
        report["validation"] = dict(fit_rows=int(fit_m.sum()), validation_rows=int(val_m.sum()), trials=trials,
                                    chosen=best)
    chosen_fit = None
    for n in sorted({4, 5, 6, 8, 15, a.n_kept}):
        if a.n_kept_batched > 0:
            kept, reg, tree = fit_by_regime(X[tr], P[tr], n, a.n_kept_batched, a.max_depth, a.min_samples_leaf,
                                            a.weighted, prune_rows[tr])
        else:
            kept, reg, tree = fit(X[tr], P[tr], n, a.max_depth, a.min_samples_leaf, a.weighted, prune_rows[tr])
        ev_tr, ev_te = evaluate(tree, kept, X[tr], P[tr], F[tr]), evaluate(tree, kept, X[te], P[te], F[te])
        per_cfg = {}
        for cfg in sorted({r["config"] for r in rows}):
            m = te & np.array([r["config"] == cfg for r in rows])
            if m.any():
                per_cfg[str(cfg)] = evaluate(tree, kept, X[m], P[m], F[m])
        report["sweep"].append(dict(n_kept=n, kept=kept.tolist(), tree_nodes=len(tree), train=ev_tr, test=ev_te,
                                    test_by_config=per_cfg))
        print("N=%2d kept=%-40s nodes=%3d | train achievable %.4f selector %.4f | test achievable %.4f "
              "selector %.4f (best single %.4f)" % (n, kept.tolist(), len(tree), ev_tr["achievable"],
                                                    ev_tr["selector"], ev_te["achievable"],
                                                    ev_te["selector"], ev_te["best_single"]))
        if len(per_cfg) > 1:
            print("      held-out by config: " + "  ".join("cfg%s: achievable %.4f selector %.4f time %.4f" % (
                c, v["achievable"], v["selector"], v["time_ratio"]) for c, v in per_cfg.items()))
        if n == a.n_kept:
            chosen_fit = (kept, reg, tree)
    kept, reg, tree = chosen_fit
    report["deployed"] = dict(n_kept=a.n_kept, kept=kept.tolist(), tree=tree_to_json(tree),
                              pruning_tree=tree_to_json(reg))
    if a.emit:
        os.makedirs(DATA, exist_ok=True)
        with open(os.path.join(DATA, "tree_%s.json" % a.dtype), "w") as f:
            json.dump(report, f, indent=1)
        trees = {}
        for dt, default in (("f32", 35), ("bf16", 5)):
            p = os.path.join(DATA, "tree_%s.json" % dt)
            if os.path.exists(p):
                trees[dt] = tree_from_json(json.load(open(p))["deployed"]["tree"])
            else:
                trees[dt] = tree_from_json([[-1, -1, -1, default, 0]])
        emit_table(trees)
        emit_kept_set(trees)
        print("wrote %s (rebuild the library to deploy it)" % os.path.relpath(TABLE_INC))
    if a.report:
        with open(a.report, "w") as f:
            json.dump(report, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
