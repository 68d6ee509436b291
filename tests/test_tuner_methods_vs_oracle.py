"""The library's top-N / k-means / PCA + k-means pruning and PCA variance spectrum (C++) against
the numpy oracle, on seeded synthetic tables and on the measured fp32 timing table.  CPU only."""
import os

import numpy as np
import pytest

import paper_2003_06795_amd.binding as ks
from oracle import selection as sel

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def tables():
    out = []
    for seed in range(3):
        r = np.random.default_rng(seed)
        P = r.random((180, 20)) * 0.3 + 0.1
        region = r.integers(0, 5, 180)
        for c in range(5):
            P[region == c, c * 3] += 1.0 + 0.2 * r.random((region == c).sum())
        out.append(sel.normalise(P))
    path = os.path.join(ROOT, "paper_2003_06795_amd", "tune", "data", "timings_f32_cfg2.csv")
    if os.path.exists(path):
        from paper_2003_06795_amd.tune import train
        rows, T = train.load_table(path, "f32")
        out.append(sel.normalise(train.perf_of(rows, T)))
    return out


@pytest.mark.parametrize("Ph", tables())
def test_methods_match_oracle(Ph):
    ratio = ks.tune_pca_variance(Ph)
    ref = sel.pca_variance_ratio(Ph)
    np.testing.assert_allclose(ratio, ref, rtol=1e-8, atol=1e-13)
    assert abs(ratio.sum() - 1.0) < 1e-12 and np.all(np.diff(ratio) <= 1e-15)
    dims = sel.components_for(ref, 0.95)
    for n in (1, 4, 6, 8, 15):
        assert ks.tune_prune_top_n(Ph, n).tolist() == sel.prune_top_n(Ph, n)
        assert ks.tune_prune_kmeans(Ph, n).tolist() == sel.prune_kmeans(Ph, n)
        assert ks.tune_prune_kmeans(Ph, n, pca_dims=dims).tolist() == sel.prune_pca_kmeans(Ph, n, dims)
        for kept in (ks.tune_prune_top_n(Ph, n), ks.tune_prune_kmeans(Ph, n)):
            assert 1 <= len(kept) <= n


def test_all_components_equal_plain_kmeans_and_bad_arguments():
    Ph = tables()[0]
    assert ks.tune_prune_kmeans(Ph, 5, pca_dims=Ph.shape[1]).tolist() == ks.tune_prune_kmeans(Ph, 5).tolist()
    with pytest.raises(ks.KsError):
        ks.tune_prune_kmeans(Ph, 5, pca_dims=Ph.shape[1] + 1)
    with pytest.raises(ks.KsError):
        ks.tune_prune_top_n(Ph, 0)
    with pytest.raises(ks.KsError):
        ks.tune_pca_variance(np.ones((4, 3)))
