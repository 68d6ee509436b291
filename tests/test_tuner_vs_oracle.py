"""The library's C++ tuner (normalise, prune, score, fit selector, predict) against the numpy
oracle of the same pipeline, on seeded synthetic timing tables.  CPU only."""
import numpy as np
import pytest

import paper_2003_06795_amd.binding as ks
from oracle import selection as sel


def table(rows, cols, seed, structured=True):
    r = np.random.default_rng(seed)
    M, N, K = (np.exp(r.uniform(np.log(16), np.log(4096), rows)).astype(np.int64) // 8 * 8 + 8 for _ in range(3))
    tA, tB = r.integers(0, 2, rows), r.integers(0, 2, rows)
    X = np.stack([ks.features(int(m), int(n), int(k), 1, int(a), int(b))
                  for m, n, k, a, b in zip(M, N, K, tA, tB)])
    P = (r.random((rows, cols)) * 0.3 + 0.1)
    if structured:
        # a few configurations that are each good in one region of the size space
        size = np.log2(X[:, 6].astype(np.float64))
        for c in range(min(cols, 6)):
            lo = 8 + 2.5 * c
            P[:, c] += np.where((size >= lo) & (size < lo + 2.5), 1.0, 0.0) * (1 + 0.3 * tA * (c % 2))
    return X, P * 1e12


def same_tree(ours, ref, leaf_key):
    """Structural equality: same splits in the same positions, same leaf payloads."""
    def walk(i, j):
        a, b = ours[i], ref[j]
        if b["feature"] == -1:
            assert a["feature"] < 0
            assert int(a["value"]) == leaf_key(b)
            return
        assert (int(a["feature"]), int(a["threshold"])) == (b["feature"], b["threshold"])
        walk(int(a["left"]), b["left"])
        walk(int(a["right"]), b["right"])
    walk(0, 0)


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("nfeat", [ks.NUM_RAW_FEATURES, ks.NUM_FEATURES])
def test_whole_pipeline_matches_oracle(seed, nfeat):
    X, P = table(220, 24, seed)
    X = X[:, :nfeat]
    Xtr, Ptr, Xte, Pte = X[:150], P[:150], X[150:], P[150:]
    Ph = ks.tune_normalise(Ptr)
    assert np.array_equal(Ph, sel.normalise(Ptr))
    Ph_te = ks.tune_normalise(Pte)
    for n_kept in (1, 4, 6, 8, 15):
        kept, reg = ks.tune_prune_tree(Xtr, Ph, n_kept)
        ref_reg = sel.fit_regression_tree(Xtr, sel.normalise(Ptr), n_kept)
        assert kept.tolist() == sel.kept_set(ref_reg)
        assert len(reg) == len(ref_reg)
        same_tree(reg, ref_reg, lambda nd: int(np.argmax(nd["value"])))
        assert ks.tune_achievable(Ph_te, kept) == pytest.approx(sel.achievable(sel.normalise(Pte), kept), rel=1e-13)
        for depth in (3, 12):
            tree = ks.tune_fit_selector(Xtr, Ptr, kept, max_depth=depth)
            ref = sel.fit_classification_tree(Xtr, sel.labels_within(Ptr, kept), max_depth=depth)
            assert len(tree) == len(ref)
            same_tree(tree, ref, lambda nd: nd["label"])
            chosen = ks.tune_predict(tree, Xte)
            assert np.array_equal(chosen, sel.predict_labels(ref, Xte))
            s = ks.tune_selector_score(Ph_te, chosen)
            assert s == pytest.approx(sel.selector_score(sel.normalise(Pte), chosen), rel=1e-13)
            assert s <= ks.tune_achievable(Ph_te, kept) + 1e-15


def test_unstructured_table_and_min_samples_leaf():
    X, P = table(120, 10, 5, structured=False)
    Ph = ks.tune_normalise(P)
    for msl in (1, 5):
        kept, reg = ks.tune_prune_tree(X, Ph, 6, min_samples_leaf=msl)
        ref = sel.fit_regression_tree(X, sel.normalise(P), 6, min_samples_leaf=msl)
        assert kept.tolist() == sel.kept_set(ref)
        same_tree(reg, ref, lambda nd: int(np.argmax(nd["value"])))
        tree = ks.tune_fit_selector(X, P, kept, max_depth=6, min_samples_leaf=msl)
        ref = sel.fit_classification_tree(X, sel.labels_within(P, kept), max_depth=6, min_samples_leaf=msl)
        same_tree(tree, ref, lambda nd: nd["label"])


def test_training_is_reproducible_byte_for_byte_and_deploys():
    X, P = table(200, 16, 9)
    Ph = ks.tune_normalise(P)
    a = ks.tune_fit_selector(X, P, ks.tune_prune_tree(X, Ph, 8)[0])
    b = ks.tune_fit_selector(X.copy(), P.copy(), ks.tune_prune_tree(X.copy(), Ph.copy(), 8)[0])
    assert a.tobytes() == b.tobytes()
    try:
        ks.set_selector(ks.F32, a)
        r = np.random.default_rng(2)
        shapes = [(int(np.exp(r.uniform(0, 13))), int(np.exp(r.uniform(0, 13))), int(np.exp(r.uniform(0, 13))),
                   1, int(r.integers(0, 2)), int(r.integers(0, 2))) for _ in range(20000)]
        F = np.stack([ks.features(*s) for s in shapes[:2000]])
        deployed = np.array([ks.select(ks.F32, *s) for s in shapes[:2000]])
        assert np.array_equal(deployed, ks.tune_predict(a, F))
    finally:
        ks.set_selector(ks.F32, None)


def test_row_weights_steer_the_classifier():
    X, P = table(100, 6, 3)
    kept = np.array([0, 1, 2], dtype=np.int32)
    y = sel.labels_within(P, kept)
    w = np.where(y == 2, 100.0, 1.0)
    plain = ks.tune_fit_selector(X, P, kept, max_depth=1)
    weighted = ks.tune_fit_selector(X, P, kept, max_depth=1, row_weight=w)
    leaves = lambda t: sorted(int(n["value"]) for n in t if n["feature"] < 0)
    assert 2 in leaves(weighted)
    assert np.array_equal(ks.tune_fit_selector(X, P, kept, max_depth=1, row_weight=np.ones(100)), plain)


def test_bad_arguments():
    X, P = table(20, 4, 0)
    with pytest.raises(ks.KsError):
        ks.tune_achievable(ks.tune_normalise(P), [9])
    with pytest.raises(ks.KsError):
        ks.tune_selector_score(ks.tune_normalise(P), np.full(20, 4))
    with pytest.raises(ks.KsError):
        ks.tune_normalise(np.zeros((3, 3)))


def test_sampled_two_stage_fit_matches_oracle_and_reads_only_timed_cells():
    from paper_2003_06795_amd.tune import sampled
    X, P = table(260, 24, 7)
    Xtr, Ptr, Xte, Pte = X[:200], P[:200], X[200:], P[200:]
    mask = np.zeros(200, dtype=bool)
    mask[np.random.default_rng(3).permutation(200)[:60]] = True
    for n_kept in (4, 8):
        kept, tree, cells = sampled.sampled_fit(Xtr, Ptr, mask, n_kept)
        ref = sel.sampled_prune_and_train(Xtr, Ptr, mask, n_kept)
        assert kept.tolist() == ref["kept"] and cells == ref["timed_cells"]
        assert cells == 60 * 24 + 140 * len(kept) < 200 * 24
        assert np.array_equal(ks.tune_predict(tree, Xte), sel.predict_labels(ref["selector"], Xte))
        # cells the procedure does not time cannot influence the result
        poisoned = Ptr.copy()
        untimed = np.ones_like(poisoned, dtype=bool)
        untimed[mask, :] = False
        untimed[:, kept] = False
        poisoned[untimed] = 1e9
        kept2, tree2, _ = sampled.sampled_fit(Xtr, poisoned, mask, n_kept)
        assert kept2.tolist() == kept.tolist()
        assert np.array_equal(ks.tune_predict(tree2, Xte), ks.tune_predict(tree, Xte))
    # with every row in stage 1 it is the full pipeline
    kept, tree, cells = sampled.sampled_fit(Xtr, Ptr, np.ones(200, dtype=bool), 6)
    full = sel.prune_and_train(Xtr, Ptr, 6)
    assert kept.tolist() == full["kept"] and cells == 200 * 24
    assert np.array_equal(ks.tune_predict(tree, Xte), sel.predict_labels(full["selector"], Xte))
    # the stage-1 draw keeps the layouts of a shape together and is reproducible
    rows = [dict(config=2, M=8 * (i // 4 + 1), N=16, K=32, batch=1) for i in range(80)]
    m1, m2 = sampled.stage1_mask(rows, 0.25, 1), sampled.stage1_mask(rows, 0.25, 1)
    assert np.array_equal(m1, m2) and m1.sum() == 20 and np.all(m1.reshape(20, 4).all(axis=1) == m1.reshape(20, 4).any(axis=1))


def test_trees_per_regime_join_under_a_batch_comparison():
    """train.fit_by_regime: the joined tree answers every row as the tree of its regime does, its
    kept set is the union, it deploys through ks_set_selector, and rows of one regime cannot
    change what the other regime's tree says."""
    from paper_2003_06795_amd.tune import train
    X, P = table(300, 16, 21)
    r = np.random.default_rng(3)
    batched = r.random(len(X)) < 0.3
    X = X.copy()
    X[batched, train.BATCH_FEATURE] = r.choice([256, 1024, 4096], int(batched.sum()))
    P = P.copy()
    P[batched, 7] += 2e12                      # the batched rows prefer a configuration of their own
    kept, reg, tree = train.fit_by_regime(X, P, 6, 3, 12, 1, False)
    k1, _, t1 = train.fit(X[~batched], P[~batched], 6, 12, 1, False)
    k2, _, t2 = train.fit(X[batched], P[batched], 3, 12, 1, False)
    assert kept.tolist() == sorted(set(k1.tolist()) | set(k2.tolist()))
    assert (int(tree[0]["feature"]), int(tree[0]["threshold"])) == (train.BATCH_FEATURE, 1)
    got = ks.tune_predict(tree, X)
    assert np.array_equal(got[~batched], ks.tune_predict(t1, X[~batched]))
    assert np.array_equal(got[batched], ks.tune_predict(t2, X[batched]))
    assert 7 in k2.tolist()
    # other batched rows leave the single-GEMM answers alone
    P2 = P.copy()
    P2[batched] = P[batched][:, ::-1]
    tree2 = train.fit_by_regime(X, P2, 6, 3, 12, 1, False)[2]
    assert np.array_equal(ks.tune_predict(tree2, X[~batched]), got[~batched])
    try:
        ks.set_selector(ks.F32, tree)
        for i in range(0, len(X), 7):
            M, N, K, b, tA, tB = (int(v) for v in X[i, :6])
            assert ks.select(ks.F32, M, N, K, b, tA, tB) == int(got[i])
    finally:
        ks.set_selector(ks.F32, None)
    # a table with one regime only falls back to the plain fit
    assert train.fit_by_regime(X[~batched], P[~batched], 6, 3, 12, 1, False)[2].tobytes() == t1.tobytes()


@pytest.mark.parametrize("seed", [21, 22])
def test_regime_pipeline_matches_the_oracle_composition(seed):
    """train.fit_by_regime (the deployed fp32 pipeline: one pruning tree and one classifier per
    regime under a batch comparison) against oracle.selection.prune_and_train_by_regime: same kept
    set, structurally the same joined tree, same answers on unseen rows."""
    from paper_2003_06795_amd.tune import train
    X, P = table(320, 16, seed)
    r = np.random.default_rng(seed)
    batched = r.random(len(X)) < 0.3
    X = X.copy()
    X[batched, train.BATCH_FEATURE] = r.choice([256, 1024, 4096], int(batched.sum()))
    P = P.copy()
    P[batched, 7] += 2e12
    P[batched, 9] += 1e12 * (X[batched, 0] > 256)
    Xtr, Ptr, Xte = X[:240], P[:240], X[240:]
    for (n1, n2, msl) in ((6, 3, 1), (15, 4, 1), (8, 8, 4)):
        kept, _, tree = train.fit_by_regime(Xtr, Ptr, n1, n2, 12, msl, False)
        ref = sel.prune_and_train_by_regime(Xtr, Ptr, n1, n2, train.BATCH_FEATURE, 12, msl)
        assert kept.tolist() == ref["kept"]
        same_tree(tree, ref["selector"], lambda nd: nd["label"])
        assert np.array_equal(ks.tune_predict(tree, Xte), sel.predict_labels(ref["selector"], Xte))
    # a planted case the composition must get right: the batched rows' best configuration is kept
    # although no single GEMM prefers it
    assert 7 in ref["kept"] and 7 not in ref["parts"][0]["kept"]


def test_performance_table_matches_the_oracle_definition():
    r = np.random.default_rng(9)
    sizes = r.integers(1, 5000, (40, 4)).astype(np.int64)
    secs = r.random((40, 7)) * 1e-3 + 1e-6
    ours = ks.tune_performance(sizes, secs)
    flops = 2.0 * sizes[:, 0] * sizes[:, 1] * sizes[:, 2] * sizes[:, 3]
    assert np.array_equal(ours, sel.performance(flops, secs))
    with pytest.raises(ks.KsError):
        ks.tune_performance(sizes, secs * 0.0)
