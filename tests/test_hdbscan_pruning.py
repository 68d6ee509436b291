"""HDBSCAN pruning (paper Section III, the density-based method of its comparison): the numpy oracle
pinned by planted clusters, by scikit-learn's implementation of the same published algorithm and by
invariants; the library's C++ implementation against the oracle."""
import numpy as np
import pytest

import paper_2003_06795_amd.binding as ks
from oracle import selection as sel


def partition(labels):
    groups = {}
    for i, v in enumerate(np.asarray(labels).tolist()):
        if v >= 0:
            groups.setdefault(v, []).append(i)
    return sorted(tuple(g) for g in groups.values())


def blobs(seed, centres, per=40, noise=8, dim=6, spread=0.05):
    r = np.random.default_rng(seed)
    pts = [r.normal(0, spread, (per, dim)) + np.asarray(c, dtype=np.float64) for c in centres]
    pts.append(r.uniform(-1, 2, (noise, dim)))
    return np.concatenate(pts)


CENTRES = [[0] * 6, [1] * 6, [0, 1, 0, 1, 0, 1]]


def test_oracle_recovers_planted_clusters_and_marks_stragglers_as_noise():
    Z = blobs(0, CENTRES)
    lab = sel.hdbscan_labels(Z, 10)
    assert lab.max() == 2
    for b in range(3):
        block = lab[b * 40:(b + 1) * 40]
        assert (block == block[0]).all() and block[0] >= 0
    assert len({lab[0], lab[40], lab[80]}) == 3
    assert (lab[120:] == -1).sum() >= 6                     # the uniform stragglers
    # labels are numbered by first member row
    assert lab[0] == 0 and lab[40] == 1 and lab[80] == 2


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_oracle_agrees_with_scikit_learn_on_the_partition(seed):
    pytest.importorskip("sklearn")
    from sklearn.cluster import HDBSCAN
    Z = blobs(seed, CENTRES + [[2, 0, 2, 0, 2, 0]], per=30 + 5 * seed, noise=6)
    for mcs, k in ((10, 10), (8, 4), (15, 5)):
        ours = sel.hdbscan_labels(Z, mcs, k)
        theirs = HDBSCAN(min_cluster_size=mcs, min_samples=k, allow_single_cluster=False, copy=True).fit(Z).labels_
        assert partition(ours) == partition(theirs), (seed, mcs, k)


def test_oracle_invariants():
    Z = blobs(5, CENTRES, per=25, noise=5)
    lab = sel.hdbscan_labels(Z, 8)
    # a permutation of the rows permutes the partition
    perm = np.random.default_rng(1).permutation(len(Z))
    lab_p = sel.hdbscan_labels(Z[perm], 8)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(len(perm))
    assert partition(lab) == partition(lab_p[inv])
    # scaling every coordinate scales every distance: same clusters
    assert partition(sel.hdbscan_labels(3.0 * Z, 8)) == partition(lab)
    # no cluster can be smaller than min_cluster_size; a table without density structure has none
    assert all(len(g) >= 8 for g in partition(lab))
    flat = np.random.default_rng(2).random((150, 20))
    assert sel.hdbscan_labels(flat, 15).max() == -1
    kept, _ = sel.prune_hdbscan(flat, 15)
    assert kept == [int(np.argmax(flat.mean(axis=0)))]


def perf_table(seed, rows=240, cols=18):
    """Normalised-performance-like rows: a few regimes, each with its own best configuration."""
    r = np.random.default_rng(seed)
    regime = r.integers(0, 4, rows)
    P = 0.2 + 0.1 * r.random((rows, cols))
    for g in range(4):
        P[regime == g, 3 * g + 1] += 1.0 + 0.05 * r.random(int((regime == g).sum()))
        P[regime == g, 3 * g + 2] += 0.8
    return P / P.max(axis=1, keepdims=True), regime


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_library_matches_the_oracle(seed):
    Phat, regime = perf_table(seed)
    for mcs, k in ((12, 12), (20, 5), (6, 3)):
        kept, lab = ks.tune_prune_hdbscan(Phat, mcs, k)
        ref_kept, ref_lab = sel.prune_hdbscan(Phat, mcs, k)
        assert np.array_equal(lab, ref_lab), (seed, mcs, k)
        assert kept.tolist() == ref_kept
    # the planted regimes are found and their winners kept
    kept, lab = ks.tune_prune_hdbscan(Phat, 12, 12)
    assert set(kept.tolist()) == {1, 4, 7, 10}
    Z = blobs(seed, CENTRES)
    assert np.array_equal(ks.tune_prune_hdbscan(Z - Z.min() + 0.1, 10)[1], sel.hdbscan_labels(Z - Z.min() + 0.1, 10))


def test_library_argument_checks_and_degenerate_tables():
    Phat, _ = perf_table(3, rows=30, cols=12)
    with pytest.raises(ks.KsError):
        ks.tune_prune_hdbscan(Phat, 1)
    kept, lab = ks.tune_prune_hdbscan(Phat[:1], 2)
    assert lab.tolist() == [-1] and kept.tolist() == [int(np.argmax(Phat[0]))]
    same = np.tile(Phat[:1], (12, 1))                       # identical rows: distances of zero
    kept, lab = ks.tune_prune_hdbscan(same, 3)
    assert kept.tolist() == [int(np.argmax(Phat[0]))]
    assert np.array_equal(lab, sel.hdbscan_labels(same, 3))
