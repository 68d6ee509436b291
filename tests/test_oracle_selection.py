"""Pins for the numpy oracle of the prune/select pipeline (oracle/selection.py): closed forms,
brute force over all partitions on tiny tables, recovery of a planted tree, the score
inequalities stated with Table I of the paper, and scikit-learn as a second opinion."""
import itertools

import numpy as np
import pytest

from oracle import selection as sel


def random_table(rows, cols, seed, lo=16, hi=4096):
    r = np.random.default_rng(seed)
    X = np.stack([r.integers(lo, hi, rows), r.integers(lo, hi, rows), r.integers(lo, hi, rows),
                  np.ones(rows, dtype=np.int64), r.integers(0, 2, rows), r.integers(0, 2, rows)], 1)
    P = (r.random((rows, cols)) + 0.05) * 1e12
    return X, P


def test_normalise_rows_peak_at_one():
    _, P = random_table(30, 9, 0)
    Ph = sel.normalise(P)
    assert np.all(Ph.max(axis=1) == 1.0) and np.all(Ph > 0) and np.all(Ph <= 1.0)
    assert np.array_equal(np.argmax(Ph, axis=1), np.argmax(P, axis=1))
    # hand example
    assert np.array_equal(sel.normalise([[2.0, 8.0, 4.0]]), [[0.25, 1.0, 0.5]])


def test_performance_definition():
    P = sel.performance([2e9, 4e9], [[1e-3, 2e-3], [1e-3, 4e-3]])
    assert np.allclose(P, [[2e12, 1e12], [4e12, 1e12]])


def test_geometric_mean_closed_forms():
    assert sel.geometric_mean([1.0, 0.25]) == pytest.approx(0.5, rel=1e-15)
    assert sel.geometric_mean([0.5, 0.5, 0.5]) == pytest.approx(0.5, rel=1e-15)
    assert sel.geometric_mean([0.9, 0.8, 0.1]) == pytest.approx((0.9 * 0.8 * 0.1) ** (1 / 3), rel=1e-14)


def test_score_inequalities():
    """selector <= achievable(kept) <= achievable(everything) = 1, and achievable is monotone."""
    _, P = random_table(40, 12, 1)
    Ph = sel.normalise(P)
    assert sel.achievable(Ph, range(12)) == pytest.approx(1.0, abs=1e-15)
    r = np.random.default_rng(0)
    order = r.permutation(12)
    prev = 0.0
    for n in range(1, 13):
        a = sel.achievable(Ph, order[:n])
        assert a >= prev - 1e-15
        prev = a
    kept = [2, 5, 7]
    chosen = np.asarray(kept)[r.integers(0, 3, 40)]
    assert sel.selector_score(Ph, chosen) <= sel.achievable(Ph, kept) + 1e-15
    best_inside = sel.labels_within(P, kept)
    assert sel.selector_score(Ph, best_inside) == pytest.approx(sel.achievable(Ph, kept), rel=1e-14)


def test_labels_within_lowest_id_on_ties():
    P = np.array([[1.0, 3.0, 3.0, 2.0], [5.0, 1.0, 1.0, 5.0]])
    assert sel.labels_within(P, [3, 1, 2]).tolist() == [1, 3]
    assert sel.labels_within(P, [0, 3]).tolist() == [3, 0]


# --------------------------------------------------------------------------- split search

def brute_force_partition(X, Y):
    """Every integer threshold of every feature; error measured as n * variance per side."""
    best = (-1.0, None)
    total = Y.shape[0] * np.var(Y, axis=0).sum()
    for f in range(X.shape[1]):
        for t in range(int(X[:, f].min()), int(X[:, f].max())):
            L = X[:, f] <= t
            e = L.sum() * np.var(Y[L], axis=0).sum() + (~L).sum() * np.var(Y[~L], axis=0).sum()
            if total - e > best[0] + 1e-9:
                best = (total - e, L.copy())
    return best


@pytest.mark.parametrize("seed", range(6))
def test_root_split_equals_brute_force(seed):
    X, P = random_table(14, 5, seed, lo=1, hi=30)
    Y = sel.normalise(P)
    gain, f, t = sel.best_regression_split(X, Y)
    bf_gain, bf_left = brute_force_partition(X, Y)
    assert gain == pytest.approx(bf_gain, rel=1e-10)
    assert np.array_equal(X[:, f] <= t, bf_left)


def test_gini_hand_example():
    X = np.array([[1], [2], [3], [4]])
    y = np.array([0, 0, 1, 1])
    gain, f, t = sel.best_classification_split(X, y, [0, 1])
    assert (f, t) == (0, 2) and gain == pytest.approx(2.0)        # 4*(1-1/2) - 0 - 0
    y = np.array([0, 1, 1, 1])
    gain, f, t = sel.best_classification_split(X, y, [0, 1])
    assert (f, t) == (0, 1) and gain == pytest.approx(4 * (1 - (1 / 16 + 9 / 16)))


def test_tie_breaks_lowest_feature_then_threshold():
    X = np.array([[1, 1], [2, 2], [3, 3], [4, 4]])
    y = np.array([0, 1, 1, 0])
    # thresholds 1 and 3 give the same gain on both (identical) features
    _, f, t = sel.best_classification_split(X, y, [0, 1])
    assert (f, t) == (0, 1)
    Y = np.array([[0.0], [1.0], [1.0], [0.0]])
    _, f, t = sel.best_regression_split(X, Y)
    assert (f, t) == (0, 1)


def planted_table():
    """Workloads on a grid whose performance vectors come from a known 3-leaf tree:
    M <= 100 -> v0 ; else K <= 50 -> v1 ; else v2."""
    Ms, Ks = [16, 40, 96, 104, 300, 900], [8, 24, 48, 56, 128, 512]
    v = np.array([[1.0, 0.2, 0.1, 0.3], [0.2, 0.1, 1.0, 0.3], [0.1, 1.0, 0.2, 0.3]])
    X, Y = [], []
    for M, N, K in itertools.product(Ms, [32, 64], Ks):
        X.append([M, N, K, 1, 0, 0])
        Y.append(v[0] if M <= 100 else (v[1] if K <= 50 else v[2]))
    return np.array(X), np.array(Y)


def test_planted_tree_is_recovered():
    X, Y = planted_table()
    tree = sel.fit_regression_tree(X, Y, max_leaf_nodes=3)
    assert len(tree) == 5
    root = tree[0]
    assert (root["feature"], root["threshold"]) == (0, 100)       # floor((96+104)/2)
    right = tree[root["right"]]
    assert (right["feature"], right["threshold"]) == (2, 52)      # floor((48+56)/2)
    assert sel.kept_set(tree) == [0, 1, 2]
    # more leaves than structure: nothing left to gain, growth stops by itself
    assert len(sel.fit_regression_tree(X, Y, max_leaf_nodes=8)) == 5
    clf = sel.fit_classification_tree(X, np.argmax(Y, axis=1))
    assert np.array_equal(sel.predict_labels(clf, X), np.argmax(Y, axis=1))
    assert sum(nd["feature"] == -1 for nd in clf) == 3


def test_leaf_limit_bounds_kept_set_and_best_first_order():
    X, P = random_table(120, 20, 3)
    Y = sel.normalise(P)
    for n in (1, 2, 5, 8, 15):
        tree = sel.fit_regression_tree(X, Y, n)
        leaves = [nd for nd in tree if nd["feature"] == -1]
        assert len(leaves) == n and len(sel.kept_set(tree)) <= n
        assert sorted(np.concatenate([nd["rows"] for nd in leaves]).tolist()) == list(range(120))
    # best-first: the n-leaf tree is a prefix of the (n+1)-leaf tree
    t5, t6 = sel.fit_regression_tree(X, Y, 5), sel.fit_regression_tree(X, Y, 6)
    for a, b in zip(t5, t6[:len(t5)]):
        assert np.array_equal(a["rows"], b["rows"])


def test_unlimited_classifier_reproduces_training_labels():
    X, P = random_table(150, 10, 4)
    kept = [1, 4, 6, 9]
    y = sel.labels_within(P, kept)
    clf = sel.fit_classification_tree(X, y, max_depth=64)
    assert np.array_equal(sel.predict_labels(clf, X), y)
    Ph = sel.normalise(P)
    assert sel.selector_score(Ph, sel.predict_labels(clf, X)) == pytest.approx(sel.achievable(Ph, kept))
    shallow = sel.fit_classification_tree(X, y, max_depth=2)
    assert max_depth_of(shallow) <= 2


def max_depth_of(tree, i=0):
    if tree[i]["feature"] == -1:
        return 0
    return 1 + max(max_depth_of(tree, tree[i]["left"]), max_depth_of(tree, tree[i]["right"]))


def test_tree_pruned_set_never_beats_exhaustive_best_subset():
    X, P = random_table(60, 9, 5)
    Ph = sel.normalise(P)
    for n in (1, 2, 3):
        kept = sel.kept_set(sel.fit_regression_tree(X, Ph, n))
        best = max(sel.achievable(Ph, c) for k in range(1, n + 1)
                   for c in itertools.combinations(range(9), k))
        assert sel.achievable(Ph, kept) <= best + 1e-15


def test_pipeline_end_to_end_on_structured_table():
    """A table with real structure: three configurations, each best in one region of sizes."""
    r = np.random.default_rng(7)
    X, _ = random_table(300, 3, 7)
    size = X[:, 0] * X[:, 1]
    P = np.empty((300, 6))
    P[:, 0] = np.where(size < 2e5, 1.0, 0.3)
    P[:, 1] = np.where((size >= 2e5) & (X[:, 2] < 1000), 1.0, 0.4)
    P[:, 2] = np.where((size >= 2e5) & (X[:, 2] >= 1000), 1.0, 0.35)
    P[:, 3:] = 0.2
    P *= 1 + 0.01 * r.random((300, 6))
    out = sel.prune_and_train(X[:200], P[:200], n_kept=6)
    assert set(out["kept"]) >= {0, 1, 2} or sel.achievable(sel.normalise(P[:200]), out["kept"]) > 0.95
    chosen = sel.predict_labels(out["selector"], X[200:])
    Ph_test = sel.normalise(P[200:])
    s, a = sel.selector_score(Ph_test, chosen), sel.achievable(Ph_test, out["kept"])
    assert s <= a + 1e-15 <= 1.0 + 1e-15 and s > 0.8


# --------------------------------------------------------------------------- second opinion

def test_sklearn_agrees_on_regression_error_and_classifier_partition():
    sk = pytest.importorskip("sklearn.tree")
    X, P = random_table(200, 16, 6)
    Y = sel.normalise(P)
    for n in (4, 8, 15):
        ours = sel.fit_regression_tree(X, Y, n)
        sse = sum(float(np.sum((Y[nd["rows"]] - nd["value"]) ** 2)) for nd in ours if nd["feature"] == -1)
        ref = sk.DecisionTreeRegressor(max_leaf_nodes=n, random_state=0).fit(X, Y)
        ref_sse = float(np.sum((ref.predict(X) - Y) ** 2))
        assert sse == pytest.approx(ref_sse, rel=1e-9)
    y = sel.labels_within(P, [0, 3, 7, 11])
    ours = sel.fit_classification_tree(X, y, max_depth=3)
    ref = sk.DecisionTreeClassifier(max_depth=3, random_state=0).fit(X, y)
    ours_leaf = np.array([sel.tree_leaf(ours, x) for x in X])
    ref_leaf = ref.apply(X)
    # same partition of the training rows into leaves (ids differ)
    pairs = set(zip(ours_leaf.tolist(), ref_leaf.tolist()))
    assert len(pairs) == len(set(ours_leaf.tolist())) == len(set(ref_leaf.tolist()))


def test_regime_composition_recovers_a_planted_two_regime_table():
    """prune_and_train_by_regime pinned by a table built from a known rule: single GEMMs (batch 1)
    prefer configuration 2 up to M = 100 and configuration 5 above, batched ones always prefer 7.
    The joined selector must be a root 'batch <= 1' over a one-split tree and a single leaf, keep
    exactly {2, 5, 7}, answer unseen rows by the rule, and a pooled tree with the same total leaf
    budget spent on the many single rows must be able to lose the batched regime's choice."""
    r = np.random.default_rng(5)
    n = 260
    M = r.integers(8, 400, n)
    batch = np.where(np.arange(n) % 13 == 0, 1024, 1)          # few batched rows
    X = np.stack([M, r.integers(8, 400, n), r.integers(8, 400, n), batch], axis=1).astype(np.int64)
    P = 0.1 + 0.05 * r.random((n, 9))
    rule = np.where(batch > 1, 7, np.where(M <= 100, 2, 5))
    P[np.arange(n), rule] = 1.0
    out = sel.prune_and_train_by_regime(X, P, 2, 1, batch_feature=3)
    assert out["kept"] == [2, 5, 7]
    root = out["selector"][0]
    assert (root["feature"], root["threshold"]) == (3, 1)
    single_root = out["selector"][root["left"]]
    assert single_root["feature"] == 0 and 93 <= single_root["threshold"] <= 107
    assert out["selector"][root["right"]]["feature"] == -1 and out["selector"][root["right"]]["label"] == 7
    Xnew = np.array([[50, 9, 9, 1], [399, 9, 9, 1], [50, 9, 9, 4096], [399, 300, 20, 256]], dtype=np.int64)
    assert sel.predict_labels(out["selector"], Xnew).tolist() == [2, 5, 7, 7]
    # the answers for single GEMMs do not depend on what the batched rows look like
    P2 = P.copy()
    P2[batch > 1] = P[batch > 1][:, ::-1]
    out2 = sel.prune_and_train_by_regime(X, P2, 2, 1, batch_feature=3)
    single = X[batch == 1]
    assert np.array_equal(sel.predict_labels(out2["selector"], single), sel.predict_labels(out["selector"], single))
    # one regime only: the plain pipeline
    only = sel.prune_and_train_by_regime(X[batch == 1], P[batch == 1], 2, 1, batch_feature=3)
    plain = sel.prune_and_train(X[batch == 1], P[batch == 1], 2)
    assert only["kept"] == plain["kept"] == [2, 5]
