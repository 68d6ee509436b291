"""GPU parity of the eight-wave 16-bit members in their two-groups-of-waves form (256 x 256 x 64:
bf16 ids 2, 20, 25 on 32x32x16 fragments, 44 and 45 on 16x16x32 fragments; 128 x 128 x 128: ids 46
and 47): against the CPU oracle within the stated bound, and bit for bit against the
generic path of the same members (same tiles, same summation order per entry).  Covers the edge
cases of that kernel's own structure: one K-step, odd and even step counts, an empty last split-K
partition, tiles whose second 128-row half lies wholly outside the matrix, all four layouts, both
16-bit operand types, padded leading dimensions and batches."""
import numpy as np
import pytest

import workloads as wl
from helpers import tolerance

pytestmark = pytest.mark.gpu

LAYOUTS = [(0, 0), (0, 1), (1, 0), (1, 1)]
PLAIN, SPLIT4, PERCALL = 2, 20, 25
PLAIN16, PERCALL16 = 44, 45           # the same form on 16x16x32 fragments
PLAIN128, PERCALL128 = 46, 47         # ... and on a 128 x 128 x 128 tile
plain_members = pytest.mark.parametrize("plain", [PLAIN, PLAIN16, PLAIN128])


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    import gpu_util
    return gpu_util


def both_paths(gpu, p, kid):
    import paper_2003_06795_amd.binding as ks
    need = ks.workspace_bytes_needed(gpu.DT[p.dtype], kid, p.M, p.N, p.batch)
    if need:
        gpu.ensure_workspace(need)
    dp = gpu.DeviceProblem(p)
    fast = dp.run(kid)
    try:
        ks.set_fast_path(False)
        slow = dp.run(kid)
    finally:
        ks.set_fast_path(True)
    return fast, slow


def check(gpu, p, kid, what):
    fast, slow = both_paths(gpu, p, kid)
    ref = gpu.oracle_full(p)
    err = float(np.max(np.abs(fast.astype(np.float64) - ref)))
    assert err <= tolerance(p), "%s: max|diff| %.3e > %.3e" % (what, err, tolerance(p))
    assert np.array_equal(fast.view(np.uint32), slow.view(np.uint32)), what + ": paths differ"


def test_members_exist_as_described(gpu):
    import paper_2003_06795_amd.binding as ks
    for kid, split, core in ((PLAIN, 1, "mfma32"), (SPLIT4, 4, "mfma32"), (PERCALL, 0, "mfma32"),
                             (PLAIN16, 1, "mfma16"), (PERCALL16, 0, "mfma16")):
        ki = ks.kernel_info(ks.BF16, kid)
        assert (ki["bm"], ki["bn"], ki["bk"], ki["wm"], ki["wn"], ki["threads"], ki["split_k"], ki["core_name"]) == \
               (256, 256, 64, 128, 64, 512, split, core)
    for kid, split in ((PLAIN128, 1), (PERCALL128, 0)):
        ki = ks.kernel_info(ks.BF16, kid)
        assert (ki["bm"], ki["bn"], ki["bk"], ki["wm"], ki["wn"], ki["threads"], ki["split_k"], ki["core_name"]) == \
               (128, 128, 128, 64, 32, 512, split, "mfma16")


@plain_members
@pytest.mark.parametrize("tA,tB", LAYOUTS)
@pytest.mark.parametrize("K", [64, 128, 192, 448, 1024, 384, 896])
def test_step_counts_and_layouts(gpu, tA, tB, K, plain):
    """1, 2, 3, 7 and 16 K-steps of 64 (1, 3, 7 and 8 of 128; K that is not a multiple of the
    member's K-step takes its general kernel); 520 x 776 spans several tiles each way with ragged edges."""
    p = wl.make_problem("bf16", tA, tB, 520, 776, K, alpha=1.0, beta=0.0, seed=31, key=K + tA * 2 + tB,
                        dist="normal", c_fill="nan")
    check(gpu, p, plain, "bf16 id %d, K %d layout %d%d" % (plain, K, tA, tB))


@plain_members
@pytest.mark.parametrize("tA,tB", LAYOUTS)
def test_second_half_of_a_tile_outside_the_matrix(gpu, tA, tB, plain):
    """M = 264 and N = 72: the last tile row keeps 8 rows (its second 128-row half is empty) and the
    only tile column keeps 72 columns; loads of absent rows are clamped, their results not stored."""
    p = wl.make_problem("bf16", tA, tB, 264, 72, 320, alpha=-1.5, beta=0.75, seed=32, key=tA * 2 + tB,
                        dist="normal", pad=(8, 16, 3))
    check(gpu, p, plain, "bf16 id %d clamped halves layout %d%d" % (plain, tA, tB))
    fast, _ = both_paths(gpu, p, plain)
    from helpers import c_padding_mask
    m = c_padding_mask(p)
    assert np.array_equal(fast[m], p.C0[m]), "padding of C was written"


@plain_members
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_batches_and_operand_types(gpu, dtype, plain):
    p = wl.make_problem(dtype, 0, 1, 512, 256, 256, batch=3, alpha=0.5, beta=-1.0, seed=33, key=5,
                        dist="normal", batch_pad=(64, 0, 8))
    check(gpu, p, plain, "%s id %d batched" % (dtype, plain))


@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1)])
def test_split_k_with_an_empty_last_partition(gpu, tA, tB):
    """K = 320 is five K-steps: four partitions get 2, 2, 1 and 0 steps."""
    p = wl.make_problem("bf16", tA, tB, 300, 520, 320, alpha=1.0, beta=0.5, seed=34, key=tB, dist="normal")
    check(gpu, p, SPLIT4, "bf16 id 20 (split 4), K 320")
    p = wl.make_problem("bf16", tA, tB, 256, 256, 8192, alpha=1.0, beta=0.0, seed=34, key=2 + tB, dist="normal",
                        c_fill="nan")
    check(gpu, p, SPLIT4, "bf16 id 20 (split 4), K 8192")
    check(gpu, p, PERCALL, "bf16 id 25 (split per call), K 8192")
    check(gpu, p, PERCALL16, "bf16 id 45 (split per call, 16x16x32 fragments), K 8192")
    check(gpu, p, PERCALL128, "bf16 id 47 (split per call, 128 x 128 x 128 tile), K 8192")


@plain_members
def test_small_integers_are_exact(gpu, plain):
    p = wl.make_problem("bf16", 0, 1, 384, 512, 704, alpha=1.0, beta=0.0, seed=35, dist="ints", c_fill="nan")
    fast, slow = both_paths(gpu, p, plain)
    assert np.array_equal(fast, gpu.oracle_full(p))
    assert np.array_equal(fast, slow)


@plain_members
def test_full_size_entries(gpu, plain):
    """4096^3 and a ragged 4104 x 4360 x 4096 in the launch bench.py times (1-D grid, XCD renumbering):
    sampled entries against the oracle."""
    import torch
    for (M, N, K, tB) in ((4096, 4096, 4096, 1), (4104, 4360, 4096, 0)):
        p = wl.make_problem("bf16", 0, tB, M, N, K, seed=36, key=M + tB, dist="normal", c_fill="zeros")
        A = torch.from_numpy(p.A.view(np.int16)).cuda()
        B = torch.from_numpy(p.B.view(np.int16)).cuda()
        C = torch.full((p.C0.size,), float("nan"), dtype=torch.float32, device="cuda")
        gpu.GEMM_K["bf16"](plain, p.transA, p.transB, M, N, K, 1.0, A, p.lda, B, p.ldb, 0.0, C, p.ldc)
        torch.cuda.synchronize()
        assert not bool(torch.isnan(C).any())
        bb, ii, jj = gpu.sample_entries(p, 2048, M)
        got = C[torch.from_numpy(ii * p.ldc + jj).cuda()].cpu().numpy()
        ref = gpu.oracle_entries(p, bb, ii, jj)
        err = float(np.max(np.abs(got.astype(np.float64) - ref.astype(np.float64))))
        assert err <= tolerance(p), "%d x %d x %d: %.3e > %.3e" % (M, N, K, err, tolerance(p))
