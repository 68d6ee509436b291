"""Pins for the oracle's other pruning methods (top-N by wins, k-means, PCA + k-means) and the PCA
variance spectrum: hand examples, planted clusters, invariants, and scikit-learn as a second
opinion where it can be driven deterministically."""
import numpy as np
import pytest

from oracle import selection as sel


def planted_clusters(seed=0, per=30, cols=12, noise=0.01):
    """Three groups of rows, each close to its own prototype vector (peaks at columns 2, 7, 9)."""
    r = np.random.default_rng(seed)
    protos = np.full((3, cols), 0.2)
    protos[0, 2] = protos[1, 7] = protos[2, 9] = 1.0
    protos[0, 7] = 0.6
    X = np.concatenate([p + noise * r.standard_normal((per, cols)) for p in protos])
    truth = np.repeat(np.arange(3), per)
    perm = r.permutation(len(X))
    return np.clip(X[perm], 0.01, None), truth[perm]


def test_top_n_hand_example():
    #            c0   c1   c2   c3
    Ph = np.array([[1.0, 0.5, 0.2, 0.1],
                   [0.3, 1.0, 0.2, 0.1],
                   [0.3, 1.0, 0.9, 0.1],
                   [0.3, 0.2, 1.0, 0.1],
                   [1.0, 1.0, 0.2, 0.1]])      # tie inside a row -> first (c0)
    # wins: c0 = 2, c1 = 2, c2 = 1, c3 = 0
    assert sel.prune_top_n(Ph, 1) == [0]               # equal counts -> lowest id
    assert sel.prune_top_n(Ph, 2) == [0, 1]
    assert sel.prune_top_n(Ph, 3) == [0, 1, 2]
    assert sel.prune_top_n(Ph, 4) == [0, 1, 2]         # a configuration that never wins is not kept


def test_kmeans_recovers_planted_clusters_and_their_best_configurations():
    X, truth = planted_clusters()
    centres, assign = sel.kmeans(X, 3)
    # same partition up to naming
    pairs = set(zip(assign.tolist(), truth.tolist()))
    assert len(pairs) == 3
    assert sel.prune_kmeans(X, 3) == [2, 7, 9]
    # centroid = mean of its rows, every row is nearest to its own centroid
    for c in range(3):
        np.testing.assert_allclose(centres[c], X[assign == c].mean(axis=0), rtol=1e-12)
    d = ((X[:, None, :] - centres[None]) ** 2).sum(axis=2)
    assert np.array_equal(np.argmin(d, axis=1), assign)


def test_kmeans_seeding_is_maximin_and_deterministic():
    Z = np.array([[0.0, 0.0], [0.1, 0.0], [10.0, 0.0], [10.0, 0.2], [0.0, 7.0], [5.0, 2.4]])
    # mean = (4.2, 1.6): closest row is (5, 2.4) -> index 5; farthest from it is (10, 0.2)? distances^2:
    # row0 30.76, row1 29.77, row2 30.76, row3 29.84, row4 46.16 -> row 4; then farthest from {5, 4}:
    # row0 min(30.76, 49) = 30.76, row2 min(30.76, 149) = 30.76 -> lowest index on the tie: row 0
    assert sel._maximin_seeds(Z, 3) == [5, 4, 0]
    a = sel.kmeans(Z, 3)
    b = sel.kmeans(Z.copy(), 3)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_kmeans_inertia_never_increases_with_more_clusters_on_nested_seeds():
    X, _ = planted_clusters(seed=3, noise=0.05)
    prev = np.inf
    for k in (1, 2, 3, 5, 8):
        centres, assign = sel.kmeans(X, k)
        inertia = float(((X - centres[assign]) ** 2).sum())
        assert inertia <= prev + 1e-9
        prev = inertia
    assert len(sel.prune_kmeans(X, 8)) <= 8


def test_kmeans_matches_sklearn_from_the_same_seeds():
    sk = pytest.importorskip("sklearn.cluster")
    r = np.random.default_rng(5)
    X = r.random((200, 10))
    k = 6
    seeds = X[sel._maximin_seeds(X, k)]
    ref = sk.KMeans(n_clusters=k, init=seeds, n_init=1, algorithm="lloyd", tol=0.0, max_iter=300).fit(X)
    centres, assign = sel.kmeans(X, k, max_iter=300)
    np.testing.assert_allclose(centres, ref.cluster_centers_, rtol=1e-9, atol=1e-12)
    assert np.array_equal(assign, ref.labels_)


def test_pca_closed_form_and_sklearn():
    # points on a line in 3-D: one component carries all the variance
    t = np.linspace(-1, 1, 21)
    X = np.stack([2 * t, -t, 0.5 * t], axis=1) + np.array([1.0, 2.0, 3.0])
    ratio = sel.pca_variance_ratio(X)
    assert ratio[0] == pytest.approx(1.0, abs=1e-12) and abs(ratio[1]) < 1e-12
    # independent axes with variances 9 : 4 : 1
    r = np.random.default_rng(0)
    Y = r.standard_normal((20000, 3)) * np.array([3.0, 2.0, 1.0])
    np.testing.assert_allclose(sel.pca_variance_ratio(Y), np.array([9, 4, 1]) / 14.0, atol=0.01)
    assert sel.components_for(np.array([0.6, 0.25, 0.1, 0.05]), 0.8) == 2
    assert sel.components_for(np.array([0.6, 0.25, 0.1, 0.05]), 0.85) == 2
    assert sel.components_for(np.array([0.6, 0.25, 0.1, 0.05]), 0.9) == 3
    skd = pytest.importorskip("sklearn.decomposition")
    Z = r.random((150, 12))
    np.testing.assert_allclose(sel.pca_variance_ratio(Z), skd.PCA().fit(Z).explained_variance_ratio_, rtol=1e-9)


def test_pca_kmeans_with_all_components_equals_plain_kmeans_and_recovers_planted():
    X, _ = planted_clusters(seed=1)
    # a rotation of the coordinates keeps every distance: same clusters, same kept set
    assert sel.prune_pca_kmeans(X, 3, X.shape[1]) == sel.prune_kmeans(X, 3) == [2, 7, 9]
    # two components already separate three clusters
    assert sel.prune_pca_kmeans(X, 3, 2) == [2, 7, 9]


def test_every_method_obeys_the_kept_set_bound_and_scores_below_one():
    r = np.random.default_rng(2)
    Ph = sel.normalise(r.random((120, 16)) + 0.05)
    for n in (1, 4, 8, 15):
        for kept in (sel.prune_top_n(Ph, n), sel.prune_kmeans(Ph, n), sel.prune_pca_kmeans(Ph, n, 5)):
            assert 1 <= len(kept) <= n and all(0 <= c < 16 for c in kept)
            assert sel.achievable(Ph, kept) <= 1.0 + 1e-15
    # top-N with N = all winners reproduces every row's best
    assert sel.achievable(Ph, sel.prune_top_n(Ph, 16)) == pytest.approx(1.0)
