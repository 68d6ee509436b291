"""The pruned library (libks_gemm_kept.so: only the kept members of the deployed trees and the four
bring-up tiles are compiled; paper Sections I, II-B, III).  It is loaded in a child process, because
a process holds one copy of the binding."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2003_06795_amd")
KEPT_LIB = os.path.join(PKG, "libks_gemm_kept.so")


def child(code, timeout=600):
    env = dict(os.environ, KS_GEMM_LIBRARY="libks_gemm_kept.so", PYTHONPATH=ROOT + os.pathsep + os.path.join(ROOT, "tests"))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, timeout=timeout, cwd=ROOT)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    return json.loads(r.stdout.strip().splitlines()[-1])


def kept_lists():
    out = {}
    for line in open(os.path.join(PKG, "csrc", "kept_set.inc")):
        if line.startswith("#define KS_KEPT_"):
            name, body = line.split(None, 2)[1:]
            out[name] = [int(v) for v in body.strip().strip("{}").split(",")]
    return out["KS_KEPT_F32"], out["KS_KEPT_BF16"]


@pytest.mark.skipif(not os.path.exists(KEPT_LIB), reason="pruned library not built (python -m paper_2003_06795_amd.build --kept-only)")
def test_pruned_library_holds_exactly_the_kept_members_and_the_selector_stays_inside():
    f32, bf16 = kept_lists()
    got = child("""
import json, numpy as np
import paper_2003_06795_amd.binding as ks
assert ks.LIB_PATH.endswith("libks_gemm_kept.so")
avail = {dt: [i for i in range(ks.num_kernels(dt)) if ks.kernel_info(dt, i)["available"]] for dt in (ks.F32, ks.BF16)}
r = np.random.default_rng(3)
picked = {ks.F32: set(), ks.BF16: set()}
for dt in picked:
    for _ in range(4000):
        M, N, K = (int(np.exp(r.uniform(0, np.log(2 ** 20)))) for _ in range(3))
        picked[dt].add(ks.select(dt, M, N, K, int(r.choice([1, 1, 1, 64, 1024])), int(r.integers(0, 2)), int(r.integers(0, 2))))
# a member that was pruned away is refused before anything is launched
absent = [i for i in range(64) if i not in avail[ks.F32]][0]
rc = ks.lib().ks_gemm_f32_with_kernel(absent, 0, 0, 8, 8, 8, 1.0, 4096, 8, 4096, 8, 0.0, 4096, 8, 1, 0, 0, 0, None)
print(json.dumps(dict(f32=avail[ks.F32], bf16=avail[ks.BF16], picked_f32=sorted(picked[ks.F32]),
                      picked_bf16=sorted(picked[ks.BF16]), rc=rc, unsupported=ks.ERR_UNSUPPORTED)))
""")
    assert got["f32"] == f32 and got["bf16"] == bf16
    assert set(got["picked_f32"]) <= set(f32) and set(got["picked_bf16"]) <= set(bf16)
    assert len(got["picked_f32"]) >= 4
    assert got["rc"] == got["unsupported"]
    assert os.path.getsize(KEPT_LIB) < 0.5 * os.path.getsize(os.path.join(PKG, "libks_gemm.so"))


@pytest.mark.gpu
def test_pruned_library_computes_the_same_gemms():
    """Selected kernels through the pruned library against the CPU oracle (fp32 and bf16, with and
    without a registered workspace, so that the twin of a fixed-split member is exercised)."""
    assert os.path.exists(KEPT_LIB), "build the pruned library first"
    got = child("""
import json, numpy as np, torch
import workloads as wl, gpu_util
from helpers import tolerance
import paper_2003_06795_amd.binding as ks
assert ks.LIB_PATH.endswith("libks_gemm_kept.so")
worst = 0.0
cases = [("f32", (200, 136, 72), 1), ("f32", (16, 24, 4096), 1), ("f32", (1000, 520, 264), 1), ("f32", (64, 64, 64), 256),
         ("f32", (2864, 2376, 840), 1), ("bf16", (264, 136, 200), 1), ("bf16", (4096, 2048, 1024), 1), ("bf16", (256, 256, 8192), 1),
         ("bf16", (64, 16, 4096), 1)]
for with_ws in (False, True):
    if with_ws:
        gpu_util.ensure_workspace(64 << 20)
    for n, (dtype, (M, N, K), batch) in enumerate(cases):
        for (tA, tB) in ((0, 0), (0, 1)):
            p = wl.make_problem(dtype, tA, tB, M, N, K, batch=batch, alpha=1.25, beta=0.5 if batch > 1 else 0.0, seed=41,
                                key=n * 2 + tB, dist="normal" if dtype == "bf16" else "uniform")
            got = gpu_util.DeviceProblem(p).run(None)
            err = float(np.max(np.abs(got.astype(np.float64) - gpu_util.oracle_full(p))))
            assert err <= tolerance(p), (dtype, M, N, K, err, tolerance(p))
            worst = max(worst, err / tolerance(p))
ks.set_workspace(None)
print(json.dumps(dict(worst=worst)))
""")
    assert got["worst"] <= 1.0
