"""The host side of a launch (ks_gemm_plan: which kernel form, how many K partitions, how many
work-groups) needs no device: the planner reads sizes, leading dimensions and pointer alignment
only.  These tests state the launch rules a second time, in Python, and compare."""
import ctypes

import pytest

import paper_2003_06795_amd.binding as ks

PTR = 1 << 20                                   # never dereferenced


@pytest.fixture()
def planner():
    L = ks.lib()
    assert L.ks_set_workspace(ctypes.c_void_p(1 << 21), ctypes.c_size_t(256 << 20)) == 0
    out = ks.LaunchPlan()

    def plan(dtype, kid, tA, tB, M, N, K, batch=1, lda=None, ldb=None, a=PTR, b=PTR, c=PTR):
        lda = lda or (M if tA else K)
        ldb = ldb or (K if tB else N)
        rc = L.ks_gemm_plan(dtype, kid, tA, tB, M, N, K, ctypes.c_float(1.0), ctypes.c_void_p(a), lda,
                            ctypes.c_void_p(b), ldb, ctypes.c_float(0.0), ctypes.c_void_p(c), N, batch,
                            M * K, K * N, M * N, ctypes.byref(out))
        assert rc == 0, rc
        return {n: int(getattr(out, n)) for n, _ in ks.LaunchPlan._fields_}
    yield plan
    ks.set_split_partitions(0)
    ks.set_balanced_groups(0)
    ks.set_tail_split(-1)
    ks.set_fast_path(True)
    L.ks_set_workspace(None, 0)


def estimate(ki, tiles, k_tiles, f32):
    """The partition count of a per-call split member, restated: work-groups run in rounds of 256 x
    (12 // waves) slots (16-bit members: at most what their LDS stages admit); a round costs the
    K-steps of a partition (times the K groups of an LDS-staged member) plus 6, partitioning costs
    10 (16-bit members: plus the partition's tile of partial sums per round); candidates fill at
    most one round (fp32: four), hold at least two steps each, and the cheapest wins, the smaller
    on ties."""
    waves = ki["threads"] // 64
    per = max(12 // waves, 1)
    if not f32 and ki["lds_bytes"] > 0:
        per = min(per, max((160 * 1024) // ki["lds_bytes"], 1))
    slots = 256 * per
    steps = -(-k_tiles // ki["k_waves"])
    smax = -(-slots // tiles)
    if f32:
        smax = max(smax, 4 * slots // tiles)
    smax = max(1, min(smax, 64 if f32 else 256))
    weight = ki["k_waves"] if ki["core_name"] != "kslice" and ki["k_waves"] > 1 else 1
    partial = 0 if f32 else (4 * ki["bm"] * ki["bn"]) // ((ki["bm"] + ki["bn"]) * ki["bk"])
    best, cost = 1, None
    for s in range(1, smax + 1):
        if s > 1 and 2 * s > steps:
            break
        c = -(-tiles * s // slots) * (weight * -(-steps // s) + 6 + (partial if s > 1 else 0)) + (10 if s > 1 else 0)
        if cost is None or c < cost:
            best, cost = s, c
    return best


@pytest.mark.parametrize("dtype", [ks.F32, ks.BF16])
def test_partition_count_of_the_per_call_split_members(planner, dtype):
    ks.set_tail_split(0)
    shapes = [(200, 136, 1024), (1184, 480, 2592), (768, 768, 3072), (96, 3016, 3392), (1408, 1256, 2560),
              (2048, 512, 2048), (312, 192, 3232), (3016, 1448, 3656), (64, 64, 8192), (1664, 896, 768)]
    seen = set()
    for kid in range(ks.num_kernels(dtype)):
        ki = ks.kernel_info(dtype, kid)
        if ki["split_k"] != 0:
            continue
        for (M, N, K) in shapes:
            tiles = -(-M // ki["bm"]) * -(-N // ki["bn"])
            want = estimate(ki, tiles, -(-K // ki["bk"]), dtype == ks.F32)
            got = planner(dtype, kid, 0, 1, M, N, K)
            assert got["split_k"] == want, (kid, (M, N, K), got, want)
            assert got["workgroups"] == tiles * want
            seen.add(want)
    assert 1 in seen and max(seen) >= 8
    # the fp32 member of 64 x 64 tiles with two K groups on 152 tiles: more partitions than fill one round
    wide = [k for k in range(ks.num_kernels(ks.F32)) if ks.kernel_info(ks.F32, k)["split_k"] == 0 and
            ks.kernel_info(ks.F32, k)["bm"] == 64 and ks.kernel_info(ks.F32, k)["threads"] == 512][0]
    assert planner(ks.F32, wide, 0, 0, 1184, 480, 2592)["split_k"] * 152 > 256


def test_forced_partitions_and_the_call_without_scratch(planner):
    kid = [k for k in range(ks.num_kernels(ks.F32)) if ks.kernel_info(ks.F32, k)["split_k"] == 0][0]
    ki = ks.kernel_info(ks.F32, kid)
    steps = -(-(-(-1000 // ki["bk"])) // ki["k_waves"])
    for forced in (1, 2, 5, 64):
        ks.set_split_partitions(forced)
        want = forced if forced == 1 or 2 * forced <= steps else max(steps // 2, 1)
        assert planner(ks.F32, kid, 0, 0, 200, 136, 1000)["split_k"] == want
    ks.set_split_partitions(0)
    for bad in (-1, 257):
        with pytest.raises(Exception):
            ks.set_split_partitions(bad)
    ks.lib().ks_set_workspace(None, 0)
    assert planner(ks.F32, kid, 0, 0, 200, 136, 4096)["split_k"] == 1


def test_balanced_persistent_form_is_taken_where_its_rule_says(planner):
    ids = [k for k in range(ks.num_kernels(ks.F32)) if ks.kernel_info(ks.F32, k)["balanced_per_cu"] > 0]
    assert ids
    for kid in ids:
        ki = ks.kernel_info(ks.F32, kid)
        bm, bn, per = ki["bm"], ki["bn"], ki["balanced_per_cu"]
        for (tm, tn, K) in ((12, 8, 1096), (13, 8, 1096), (24, 12, 3656), (24, 12, 1000), (16, 32, 2048), (64, 64, 2048),
                            (3, 1, 1024), (18, 19, 2400)):
            tiles = tm * tn
            groups = 256 * per
            if per == 2 and ki["threads"] >= 512 and tiles <= 96:
                groups = 256
            tail = tiles % groups
            takes = tail != 0 and tiles < 4 * groups and K >= 1024 and tail * -(-K // ki["bk"]) >= groups
            got = planner(ks.F32, kid, 0, 1, tm * bm - 3, tn * bn - 5, K)
            assert got["balanced_groups"] == (groups if takes else 0), (kid, tm, tn, K, got)
            assert got["divided_tiles"] == (tail if takes else 0)
            assert got["workgroups"] == (groups if takes else tiles) or got["tiles_per_workgroup"] > 1
        ks.set_balanced_groups(1)
        got = planner(ks.F32, kid, 0, 0, 24 * bm, 12 * bn, 200)          # forced: also with a short K
        assert got["balanced_groups"] == 256 and got["divided_tiles"] == 288 - 256
        ks.set_balanced_groups(0)


def test_hybrid_launch_and_cut_of_k_for_the_16_bit_members(planner):
    big = [k for k in range(ks.num_kernels(ks.BF16)) if ks.kernel_info(ks.BF16, k)["split_k"] == 0 and
           ks.kernel_info(ks.BF16, k)["bm"] == 256 and ks.kernel_info(ks.BF16, k)["bn"] == 256][-1]
    got = planner(ks.BF16, big, 0, 1, 17 * 256, 17 * 256, 8192)          # 289 tiles: one round of 256 and 33 more
    assert got["tail_split"] == 7 and got["workgroups"] == 256 + 33 * 7 and got["split_k"] == 1
    ks.set_tail_split(0)
    got = planner(ks.BF16, big, 0, 1, 17 * 256, 17 * 256, 8192)
    assert got["tail_split"] == 0 and got["workgroups"] == 289
    ks.set_tail_split(-1)
    assert planner(ks.BF16, big, 0, 1, 16 * 256, 16 * 256, 8192)["tail_split"] == 0      # nothing left over
    # K = 4104 = 64 K-steps of 64 and 8 more: the remainder runs first, through the general kernel
    got = planner(ks.BF16, big, 0, 0, 4096, 4096, 4104)
    assert got["k_remainder"] == 8 and got["path"] >= 1
    ks.set_fast_path(False)
    got = planner(ks.BF16, big, 0, 0, 4096, 4096, 4104)
    assert got["k_remainder"] == 0 and got["path"] == 0
    ks.set_fast_path(True)
    assert planner(ks.BF16, big, 0, 1, 1024, 1024, 4104)["k_remainder"] == 0             # K-contiguous pair, small output
    assert planner(ks.BF16, big, 0, 0, 4096, 4096, 4100)["k_remainder"] == 0             # K not a multiple of 8
    assert planner(ks.BF16, big, 0, 0, 4096, 4096, 4096)["path"] >= 1
    assert planner(ks.BF16, big, 0, 0, 4096, 4096, 4096, a=PTR + 2)["path"] == 0         # misaligned operand


def test_vector_loads_and_launch_shape(planner):
    kid = [k for k in range(ks.num_kernels(ks.F32)) if ks.kernel_info(ks.F32, k)["core_name"] == "mfma32" and
           ks.kernel_info(ks.F32, k)["split_k"] == 1 and ks.kernel_info(ks.F32, k)["balanced_per_cu"] == 0][0]
    assert planner(ks.F32, kid, 0, 0, 256, 256, 256)["vector_loads"] == 1
    assert planner(ks.F32, kid, 0, 0, 256, 256, 256, lda=258)["vector_loads"] == 0       # rows not 16-byte aligned
    assert planner(ks.F32, kid, 0, 0, 256, 256, 256, a=PTR + 4)["vector_loads"] == 0
    assert planner(ks.F32, kid, 0, 0, 256, 256, 256)["grid_3d"] == 1                     # few work-groups, small operands
    assert planner(ks.F32, kid, 0, 0, 4096, 4096, 256)["grid_3d"] == 0
    got = planner(ks.F32, kid, 0, 0, 256, 256, 256, batch=3)
    ki = ks.kernel_info(ks.F32, kid)
    assert got["workgroups"] == 3 * -(-256 // ki["bm"]) * -(-256 // ki["bn"])
    assert planner(ks.F32, -1, 0, 0, 256, 256, 256)["kernel_id"] == ks.select(ks.F32, 256, 256, 256, 1, 0, 0)
