"""ks_gemm_with_workspace: the scratch is an argument of the call, the registered workspace is not
touched.  Bit-identical to the registered-workspace entry points on members that split K in every
way the family knows (fixed, per call, balanced persistent form), checked against the oracle, and
the no-scratch fallbacks."""
import numpy as np
import pytest

import workloads as wl
from helpers import tolerance

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    import gpu_util
    return gpu_util


def members(ks, dt):
    """One fixed-split, one per-call-split and (fp32) one balanced member."""
    out = {}
    for i in range(ks.num_kernels(dt)):
        ki = ks.kernel_info(dt, i)
        kind = "balanced" if ki["balanced_per_cu"] > 0 else "fixed" if ki["split_k"] > 1 else \
            "per_call" if ki["split_k"] == 0 else None
        if kind and kind not in out:
            out[kind] = i
    return out


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scratch_as_an_argument_equals_the_registered_workspace(gpu, dtype):
    import torch
    import paper_2003_06795_amd.binding as ks
    dt = gpu.DT[dtype]
    p = wl.make_problem(dtype, 0, 1, 392, 264, 4096, alpha=1.25, beta=0.5, seed=51,
                        dist="normal" if dtype == "bf16" else "uniform")
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    args = (p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta)
    tail = (p.ldc, )
    found = members(ks, dt)
    assert "fixed" in found and "per_call" in found and (dtype != "f32" or "balanced" in found)
    for kind, kid in found.items():
        need = ks.workspace_bytes_needed(dt, kid, p.M, p.N, p.batch)
        assert need > 0
        gpu.ensure_workspace(need)
        registered = dp.run(kid)
        assert float(np.max(np.abs(registered.astype(np.float64) - ref))) <= tolerance(p), (kind, kid)
        mine = torch.empty(need // 4 + 1, dtype=torch.float32, device="cuda")
        try:
            ks.set_workspace(None)                     # nothing registered: only the argument can serve
            C = dp.C0.clone()
            ks.gemm_with_workspace(dt, kid, *args, C, *tail, mine)
            torch.cuda.synchronize()
            assert np.array_equal(C.cpu().numpy(), registered), "%s member %d differs" % (kind, kid)
            # without scratch: a fixed split is refused and launches nothing, the others run unsplit
            C2 = dp.C0.clone()
            if kind == "fixed":
                with pytest.raises(ks.KsError) as e:
                    ks.gemm_with_workspace(dt, kid, *args, C2, *tail, None)
                assert e.value.status == ks.ERR_WORKSPACE
                torch.cuda.synchronize()
                assert torch.equal(C2, dp.C0)
            else:
                ks.gemm_with_workspace(dt, kid, *args, C2, *tail, None)
                torch.cuda.synchronize()
                assert float(np.max(np.abs(C2.cpu().numpy().astype(np.float64) - ref))) <= tolerance(p)
        finally:
            gpu.ensure_workspace.__defaults__[0].clear()


def test_selected_kernel_with_scratch_argument(gpu):
    import torch
    import paper_2003_06795_amd.binding as ks
    p = wl.make_problem("f32", 0, 0, 96, 3016, 3392, alpha=1.0, beta=0.0, seed=52, c_fill="nan")
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    mine = torch.empty(16 << 20, dtype=torch.float32, device="cuda")
    C = dp.C0.clone()
    ks.gemm_with_workspace(ks.F32, -1, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta,
                           C, p.ldc, mine)
    torch.cuda.synchronize()
    assert float(np.max(np.abs(C.cpu().numpy().astype(np.float64) - ref))) <= tolerance(p)
    # a null scratch pointer with a size, or a misaligned one, is refused before anything is launched
    raw = ks.lib().ks_gemm_with_workspace
    common = (ks.F32, -1, 0, 0, 8, 8, 8, 1.0, dp.A.data_ptr(), 8, dp.B.data_ptr(), 8, 0.0, C.data_ptr(), 8, 1, 0, 0, 0)
    assert raw(*common, None, 64, None) == ks.ERR_INVALID_ARG
    assert raw(*common, mine.data_ptr() + 2, 64, None) == ks.ERR_INVALID_ARG
    assert raw(*common, mine.data_ptr(), 0, None) == ks.ERR_INVALID_ARG
