#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg5|fp32_large] [--single-launch]

A step is one pass of the deployed library over the workload: for every (shape, layout) row,
ks_select picks a kernel and ks_gemm_* runs it (inputs resident in HBM).  The default workload is
the fp32 tuning set (200 log-uniform shapes x 4 layouts = 800 GEMMs); `value` is the geometric
mean over rows of TFLOP/s, each row's time being the median over the K timed steps of the HIP
event interval around its launch.  One JSON line is printed.  Besides the contract's fields it
carries, all measured in the same run after the timed region:
  roofline       the single-kernel GEMM symbol that does the most flops in a pass
  selector       stored held-out score and a live one: every kernel timed on seeded held-out rows
  fp32_large     4096^3 in four layouts and three large im2col rows, fraction of the fp32 matrix peak
  cfg3_sample, cfg4   geometric means over an im2col sample and the 64 batched small shapes
  bf16_large     the large / skinny bf16 cells, fraction of the bf16 matrix peak and of what a pure
                 MFMA loop sustains on the same operand values (ks_mfma_sustained)
  cpu_baseline   the CPU oracle on a bounded sample of the same rows
--single-launch makes every sample one launch (what a profiler run wants: each row then
contributes the same number of launches to its kernel symbol's average).
"""
import argparse
import json
import os
import platform
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"f32": 157.3, "bf16": 2516.6}      # dense matrix-core TFLOP/s of MI355X
HBM_TBS = 8.0                              # published HBM3E bandwidth, TB/s
CALIB_BYTES = 256 * 1024 * 1024
SAMPLES = 3                                 # timed samples per row per step


def attainable_tflops(dtype, M, N, K, batch=1, beta=0.0):
    """Roofline bound of one GEMM: min(matrix peak, arithmetic intensity x HBM bandwidth), with the
    algorithmic bytes (each operand once, C written once and read once if beta != 0)."""
    esz = 4 if dtype == "f32" else 2
    by = batch * ((M * K + K * N) * esz + M * N * 4 * (2 if beta != 0.0 else 1))
    return min(PEAK[dtype], 2.0 * M * N * K * batch / by * HBM_TBS)


def kernel_symbol(ks, dt, plan, tA, tB):
    """Name of the device function a call resolves to (as rocprofv3 prints it), from what the
    library says it would launch (ks_gemm_plan): member, split actually taken, code path."""
    ki = ks.kernel_info(dt, plan["kernel_id"])
    akc, bkc = int(not tA), int(bool(tB))
    split, vec = plan["split_k"] > 1, plan["vector_loads"]
    b = lambda v: "true" if v else "false"
    if dt == ks.F32 and ki["core_name"] == "direct":
        return "gemm_f32_direct_kernel<%d, %d, %d, %d, %d, %s, %s, %s, %s>" % (
            ki["bm"], ki["bn"], ki["bk"], ki["wm"], ki["wn"], b(split), b(akc), b(bkc), b(vec))
    if dt == ks.F32 and ki["core_name"] == "kslice":
        return "gemm_f32_kslice_kernel<%d, %d, %d, %d, %d, %s, %s, %s, %s>" % (
            ki["bm"], ki["bn"], ki["bk"], ki["k_waves"], ki["wm"], b(split), b(akc), b(bkc), b(vec))
    if dt == ks.F32:
        p1, p2 = (ki["tm"], ki["tn"]) if ki["core_name"] == "fma" else (ki["wm"], ki["wn"])
        return "gemm_f32_kernel<%d, %d, %d, %d, %d, %d, %s, %s, %s, %s, %d, %s, %s>" % (
            ki["core"], ki["bm"], ki["bn"], ki["bk"], p1, p2, b(split), b(akc), b(bkc), b(vec), ki["k_waves"],
            b(plan["tiles_per_workgroup"] > 1), b(plan["balanced_groups"] > 0))
    f = 16 if ki["core_name"] == "mfma16" else 32
    if plan["path"] == 2:
        return "gemm_bf16_pp_kernel<%d, %s, %s, %s, false, 0, %d, %d>" % (f, b(split), b(akc), b(bkc), ki["bm"], ki["bk"])
    if plan["path"] == 1:
        stages = ki["lds_bytes"] // (ki["bk"] * (ki["bm"] + ki["bn"]) * 2)
        return "gemm_bf16_dma_kernel<%d, %d, %d, %d, %d, %d, %d, %s, %s, %s, false>" % (
            f, ki["bm"], ki["bn"], ki["bk"], ki["wm"], ki["wn"], stages, b(split), b(akc), b(bkc))
    return "gemm_bf16_kernel<%d, %d, %d, %d, %d, %d, %s, %s, %s, %s, false>" % (
        f, ki["bm"], ki["bn"], ki["bk"], ki["wm"], ki["wn"], b(split), b(akc), b(bkc), b(vec))


def build_rows(workload):
    import workloads as wl
    rows = []
    if workload == "cfg2":
        for (s, tA, tB, M, N, K, b) in wl.config2_rows():
            rows.append(dict(dtype="f32", shape=s, tA=tA, tB=tB, M=M, N=N, K=K, batch=b, alpha=1.0, beta=0.0))
    elif workload == "cfg5":
        for s, (M, N, K) in enumerate(wl.config5_shapes()):
            for (tA, tB) in wl.CONFIG5_LAYOUTS:
                rows.append(dict(dtype="bf16", shape=s, tA=tA, tB=tB, M=M, N=N, K=K, batch=1, alpha=1.0, beta=0.0))
    elif workload == "cfg4":
        for s, (M, N, K) in enumerate(wl.config4_shapes()):
            rows.append(dict(dtype="f32", shape=s, tA=0, tB=0, M=M, N=N, K=K, batch=wl.CONFIG4_BATCH,
                             alpha=wl.CONFIG4_ALPHA, beta=wl.CONFIG4_BETA))
    elif workload == "cfg3_sample":
        shapes = wl.config3_shapes()
        pick = np.random.default_rng(3).choice(len(shapes), 64, replace=False)
        for s in sorted(int(i) for i in pick):
            M, N, K = shapes[s]
            if (M * K + K * N + M * N) * 4 > 6e9:          # keeps the sample's footprint bounded
                continue
            rows.append(dict(dtype="f32", shape=s, tA=0, tB=0, M=M, N=N, K=K, batch=1, alpha=1.0, beta=0.0))
    elif workload == "fp32_large":
        for s, (M, N, K) in enumerate([(4096, 4096, 4096), (100352, 2048, 4608), (25088, 512, 1152),
                                       (401408, 2048, 32)]):
            for (tA, tB) in (((0, 0), (0, 1), (1, 0), (1, 1)) if s == 0 else ((0, 0),)):
                rows.append(dict(dtype="f32", shape=s, tA=tA, tB=tB, M=M, N=N, K=K, batch=1, alpha=1.0, beta=0.0))
    else:
        raise SystemExit("unknown workload %r" % workload)
    return rows


def allocate(rows, torch):
    """One (A, B, C) set per distinct shape; the layouts of a shape reinterpret the same buffers."""
    g = torch.Generator(device="cuda")
    bufs = {}
    for r in rows:
        key = (r["dtype"], r["shape"])
        if key in bufs:
            continue
        g.manual_seed(1000 + r["shape"])
        M, N, K, b = r["M"], r["N"], r["K"], r["batch"]
        if r["dtype"] == "f32":
            A = torch.rand(M * K * b, generator=g, device="cuda") * 2 - 1
            B = torch.rand(K * N * b, generator=g, device="cuda") * 2 - 1
        else:
            s = 1.0 / np.sqrt(K)
            A = (torch.randn(M * K * b, generator=g, device="cuda") * s).to(torch.bfloat16)
            B = (torch.randn(K * N * b, generator=g, device="cuda") * s).to(torch.bfloat16)
        C = (torch.rand(M * N * b, generator=g, device="cuda") * 2 - 1) if r["beta"] != 0.0 else \
            torch.zeros(M * N * b, device="cuda")
        bufs[key] = (A, B, C)
    return bufs


def gemm_args(r, bufs):
    A, B, C = bufs[(r["dtype"], r["shape"])]
    M, N, K, b = r["M"], r["N"], r["K"], r["batch"]
    return (r["tA"], r["tB"], M, N, K, r["alpha"], A, M if r["tA"] else K, B, K if r["tB"] else N, r["beta"], C, N,
            b, M * K if b > 1 else 0, K * N if b > 1 else 0, M * N if b > 1 else 0)


def reps_of(rows, single):
    """Launches per sample: about 1.2e9 flops, at most 64 (roughly the tuner's 100 us samples), a
    fixed function of the row so that warm-up and timed passes launch exactly the same kernels."""
    if single:
        return [1] * len(rows)
    return [int(min(64, max(1, np.ceil(1.2e9 / (2.0 * r["M"] * r["N"] * r["K"] * r["batch"]))))) for r in rows]


def run_pass(ks, rows, bufs, reps, stream, out_ms=None, kernel=-1):
    """One pass: every row's GEMM with the selected kernel (kernel id -1 = ks_select), timed the way
    the tuner times a cell (ks_time_gemm): one untimed launch, then SAMPLES samples of reps[i]
    back-to-back launches, each between one HIP event pair.  The untimed launch keeps the queue
    ahead of the device, so a sample measures kernel time and not the host's enqueue rate.
    out_ms[i] receives the median per-launch milliseconds of the samples."""
    for i, r in enumerate(rows):
        ms = ks.time_gemm(ks.F32 if r["dtype"] == "f32" else ks.BF16, kernel, *gemm_args(r, bufs),
                          stream=stream, warmup=1, iters=SAMPLES, reps=reps[i])
        if out_ms is not None:
            out_ms[i] = float(np.median(ms))


def ensure_workspace(ks, torch, nbytes, _state={}):
    if nbytes > _state.get("bytes", 0):
        _state["buf"] = torch.empty(nbytes // 4 + 1, dtype=torch.float32, device="cuda")
        _state["bytes"] = nbytes
    if "buf" in _state:
        ks.set_workspace(_state["buf"])


def workspace_for(ks, torch, rows):
    need = 0
    for r in rows:
        dt = ks.F32 if r["dtype"] == "f32" else ks.BF16
        kid = ks.select(dt, r["M"], r["N"], r["K"], r["batch"], r["tA"], r["tB"])
        need = max(need, ks.workspace_bytes_needed(dt, kid, r["M"], r["N"], r["batch"]))
    ensure_workspace(ks, torch, need)


def flops_of(rows):
    return np.array([2.0 * r["M"] * r["N"] * r["K"] * r["batch"] for r in rows])


def stored_traffic(workload, symbol):
    """HBM bytes per launch of `symbol` from the committed counter summary (two rocprofv3 --pmc runs
    of this script, FETCH_SIZE and WRITE_SIZE, scaled by the calibration copy), or None."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic_%s.txt" % workload)
    if not os.path.exists(path):
        return None
    for k in json.load(open(path)).get("kernels", []):
        if k["kernel"] == symbol or k["kernel"].startswith(symbol.rstrip(">")):
            return dict(fetch_bytes=k["fetch_bytes"], write_bytes=k["write_bytes"],
                        total_bytes=k["fetch_bytes"] + k["write_bytes"], algorithmic_bytes=k.get("algorithmic_bytes"))
    return None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return platform.processor() or "unknown"


def cpu_baseline(rows, budget_s=12.0):
    """The CPU oracle, as it stands, on a seeded sample of the same rows (small ones first so the
    sample is bounded); geometric mean of its TFLOP/s over the sampled rows with all the threads
    OpenMP gives it, and again on the first rows of the sample with one thread."""
    import workloads as wl
    from oracle import gemm as og
    order = np.random.default_rng(0).permutation(len(rows))
    threads = og.num_threads()

    def timed(i):
        r = rows[int(i)]
        p = wl.make_problem(r["dtype"], r["tA"], r["tB"], r["M"], r["N"], r["K"], batch=r["batch"],
                            alpha=r["alpha"], beta=r["beta"], seed=1, key=int(i),
                            dist="normal" if r["dtype"] == "bf16" else "uniform")
        C = p.C0.copy()
        t0 = time.perf_counter()
        og.gemm(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, C,
                p.ldc, p.batch, p.strideA, p.strideB, p.strideC)
        return time.perf_counter() - t0

    picked, rates, spent = [], [], 0.0
    for i in order:
        r = rows[int(i)]
        macs = r["M"] * r["N"] * r["K"] * r["batch"]
        if macs > 2 ** 34 or spent > budget_s:
            continue
        dt = timed(i)
        spent += dt
        picked.append(int(i))
        rates.append(2.0 * macs / dt / 1e12)
        if len(picked) >= 400:
            break
    # one thread: the same rows in the same order until a third of the budget is spent
    og.set_num_threads(1)
    rates1, spent1 = [], 0.0
    try:
        for i in picked:
            r = rows[i]
            macs = r["M"] * r["N"] * r["K"] * r["batch"]
            if macs > 2 ** 30 or spent1 > budget_s / 3:
                continue
            dt = timed(i)
            spent1 += dt
            rates1.append(2.0 * macs / dt / 1e12)
    finally:
        og.set_num_threads(threads)
    gm = lambda v: float(np.exp(np.mean(np.log(v)))) if len(v) else None
    return dict(value=gm(rates), unit="TFLOP/s (geomean over sampled rows)", cores=threads, kind="oracle",
                cpu=cpu_model(),
                sample="%d seeded rows of the workload with M*N*K <= 2^34, full fp64 triple loop, %.1f s of CPU work"
                       % (len(picked), spent),
                one_thread=dict(value=gm(rates1), cores=1,
                                sample="%d of those rows with M*N*K <= 2^30, %.1f s" % (len(rates1), spent1)))


def frac_summary(tflops, rows):
    """Achieved / min(peak, AI x 8 TB/s) per row: geometric mean, quartiles and the maximum.  Most rows
    of the fp32 tuning set last a few microseconds, where launch latency (not in this bound) rules."""
    f = np.array([t / attainable_tflops(r["dtype"], r["M"], r["N"], r["K"], r["batch"], r["beta"])
                  for t, r in zip(tflops, rows)])
    q = np.quantile(f, [0.25, 0.5, 0.75])
    return dict(geomean=float(np.exp(np.mean(np.log(f)))), q25=float(q[0]), median=float(q[1]),
                q75=float(q[2]), max=float(f.max()))


def time_set(ks, torch, workload, iters=10):
    """Selected kernels on a named shape set, after the timed region: per-cell TFLOP/s."""
    rows = build_rows(workload)
    cells = []
    # one shape at a time: the large im2col rows hold several GB
    for key in sorted({r["shape"] for r in rows}):
        sub = [r for r in rows if r["shape"] == key]
        bufs = allocate(sub, torch)
        workspace_for(ks, torch, sub)
        for r in sub:
            dt = ks.F32 if r["dtype"] == "f32" else ks.BF16
            args = gemm_args(r, bufs)
            plan = ks.gemm_plan(dt, -1, *args)
            fl = 2.0 * r["M"] * r["N"] * r["K"] * r["batch"]
            reps = int(min(64, max(1, np.ceil(1.2e9 / fl))))
            # the clock the device holds settles over some tens of milliseconds of load (the first
            # cell measured after the buffers were filled reads several per cent low otherwise):
            # a first estimate sizes about 30 ms of untimed launches before the timed samples
            est = float(np.median(ks.time_gemm(dt, -1, *args, warmup=1, iters=3, reps=reps)))
            warm = int(min(64, max(2, np.ceil(30.0 / max(est * reps, 1e-3)))))
            t = float(np.median(ks.time_gemm(dt, -1, *args, warmup=warm, iters=iters, reps=reps)))
            tf = fl / (t * 1e-3) / 1e12
            att = attainable_tflops(r["dtype"], r["M"], r["N"], r["K"], r["batch"], r["beta"])
            cells.append(dict(M=r["M"], N=r["N"], K=r["K"], batch=r["batch"], layout="NT"[r["tA"]] + "NT"[r["tB"]],
                              kernel=plan["kernel_id"], split_k=plan["split_k"], tail_split=plan["tail_split"], ms=t,
                              tflops=tf,
                              frac_of_peak=tf / PEAK[r["dtype"]], attainable_tflops=att, frac_of_attainable=tf / att))
        del bufs
        torch.cuda.empty_cache()
    return cells


SUSTAINED_FLOPS = 3e8          # rows of at least this many flops are timed again under sustained load


def sustained_clock_report(ks, rows, bufs, reps, med, flops, dtype, probe, mhz_after_pass):
    """The shader clock follows the load: after idle or a stretch of launch-bound GEMMs it sits
    near 2.1 GHz and takes some tens of milliseconds of full load to reach the 2.4 GHz the
    published peak assumes.  Inside a pass a large row gets four launches between rows of a few
    microseconds, so it is timed at the lower clock; the tuner's tables (64 kernels in a row on one
    shape) and the cells measured beside the timed region are taken at the sustained one.  This
    re-times the rows of >= SUSTAINED_FLOPS flops back to back, after 30 ms of load, and reports
    what the pass would take with those rows at the sustained clock (the others as timed)."""
    dt = ks.F32 if dtype == "f32" else ks.BF16
    big = [i for i in range(len(rows)) if flops[i] >= SUSTAINED_FLOPS]
    if not big:
        return None
    i0 = max(big, key=lambda i: flops[i])
    n0 = int(min(256, max(2, np.ceil(30.0 / max(med[i0], 1e-3)))))
    ks.time_gemm(dt, -1, *gemm_args(rows[i0], bufs), warmup=n0, iters=1, reps=1)
    hot = np.array(med, dtype=np.float64)
    for i in sorted(big, key=lambda i: -flops[i]):
        hot[i] = float(np.median(ks.time_gemm(dt, -1, *gemm_args(rows[i], bufs), warmup=2, iters=5, reps=reps[i])))
    _, mhz_hot = ks.mfma_sustained(dt, probe, rounds=20)
    t_pass, t_hot = float(med.sum() * 1e-3), float(hot.sum() * 1e-3)
    return dict(rows_timed_again=len(big), flops_at_least=SUSTAINED_FLOPS,
                their_ms_in_the_pass=float(med[big].sum()), their_ms_under_sustained_load=float(hot[big].sum()),
                device_ms=t_hot * 1e3, tflops=float(flops.sum() / t_hot / 1e12),
                frac_of_peak=float(flops.sum() / t_hot / 1e12 / PEAK[dtype]),
                value_with_those_rows=geomean(flops / (hot * 1e-3) / 1e12),
                shader_mhz=dict(after_the_timed_passes=mhz_after_pass, after_these_rows=mhz_hot,
                                how="ks_mfma_sustained, 20 rounds (0.3 ms per launch, second of two launches)"),
                what=("the pass with its rows of >= %.0e flops timed again back to back after 30 ms of load "
                      "(2 untimed launches, median of 5 samples); the other rows as in the pass" % SUSTAINED_FLOPS))


def geomean(v):
    return float(np.exp(np.mean(np.log(np.asarray(v, dtype=np.float64)))))


def selector_live(ks, torch, n_shapes=6):
    """Section III-A / Table I measured in this run: every one of the 64 fp32 kernels timed on seeded
    held-out rows of the tuning set (shapes the deployed tree never saw), and the geometric mean of
    time(best kernel) / time(selected kernel)."""
    import workloads as wl
    held = wl.config2_split()[1]
    pick = sorted(int(s) for s in np.random.default_rng(7).choice(held, n_shapes, replace=False))
    rows = [r for r in build_rows("cfg2") if r["shape"] in pick]
    bufs = allocate(rows, torch)
    nk = ks.num_kernels(ks.F32)
    need = 0
    for r in rows:
        for k in range(nk):
            need = max(need, ks.workspace_bytes_needed(ks.F32, k, r["M"], r["N"], r["batch"]))
    ensure_workspace(ks, torch, min(need, 1 << 30))
    reps = reps_of(rows, False)
    ratios, detail = [], []
    for i, r in enumerate(rows):
        args = gemm_args(r, bufs)
        sel = ks.gemm_plan(ks.F32, -1, *args)["kernel_id"]
        t = np.full(nk, np.inf)
        for k in range(nk):
            try:
                t[k] = float(np.median(ks.time_gemm(ks.F32, k, *args, warmup=1, iters=SAMPLES, reps=reps[i])))
            except ks.KsError:
                pass                                  # a fixed-split member beyond the workspace
        best = int(np.argmin(t))
        ratios.append(t[best] / t[sel])
        detail.append(dict(M=r["M"], N=r["N"], K=r["K"], layout="NT"[r["tA"]] + "NT"[r["tB"]], selected=sel,
                           best=best, ratio=float(t[best] / t[sel])))
    return dict(rows=len(rows), kernels_timed=nk, held_out_shapes=pick,
                selected_over_best_geomean=geomean(ratios), worst=min(detail, key=lambda d: d["ratio"]))


def bf16_launch_forms(ks, torch):
    """The launch forms the named cells never take (their sizes are powers of two), each against the
    form it replaces, on the selected kernel: a partly filled last round of tiles cut along K
    (ks_set_tail_split) and a K that is not a whole number of K-steps (ks_set_fast_path)."""
    out = []
    for (M, N, K, tA, tB, what) in ((4352, 4352, 8192, 0, 1, "hybrid"), (4160, 4160, 4096, 0, 1, "hybrid"),
                                    (4096, 4096, 4104, 0, 0, "cut_k"), (1024, 1024, 1032, 1, 0, "cut_k")):
        s = 1.0 / np.sqrt(K)
        A = (torch.randn(M * K, device="cuda") * s).to(torch.bfloat16)
        B = (torch.randn(K * N, device="cuda") * s).to(torch.bfloat16)
        C = torch.zeros(M * N, device="cuda")
        args = (tA, tB, M, N, K, 1.0, A, M if tA else K, B, K if tB else N, 0.0, C, N)
        ws = ensure_workspace(ks, torch, 256 << 20)
        t = {}
        for on in (True, False):
            if what == "hybrid":
                ks.set_tail_split(-1 if on else 0)
            else:
                ks.set_fast_path(on)
            plan = ks.gemm_plan(ks.BF16, -1, *args)
            est = float(np.median(ks.time_gemm(ks.BF16, -1, *args, warmup=1, iters=3, reps=1)))
            warm = int(min(64, max(2, np.ceil(30.0 / max(est, 1e-3)))))
            t[on] = (float(np.median(ks.time_gemm(ks.BF16, -1, *args, warmup=warm, iters=8, reps=1))), plan)
        ks.set_tail_split(-1)
        ks.set_fast_path(True)
        fl = 2.0 * M * N * K
        out.append(dict(M=M, N=N, K=K, layout="NT"[tA] + "NT"[tB], form=what, kernel=t[True][1]["kernel_id"],
                        tail_split=t[True][1]["tail_split"], k_remainder=t[True][1]["k_remainder"],
                        ms=t[True][0], tflops=fl / (t[True][0] * 1e-3) / 1e12,
                        ms_in_the_form_it_replaces=t[False][0], speedup=t[False][0] / t[True][0]))
        del A, B, C, ws
    return out


def f32_launch_forms(ks, torch):
    """The launch shape as the run-time axis on the fp32 side, each form against the one it replaces
    on the kernel the deployed tree selects: the balanced persistent form against the plain launch of
    the same member (ks_set_workspace: without scratch the member runs plain), and the K partition
    count the library's estimate takes against no partitioning (ks_set_split_partitions)."""
    out = []
    for (M, N, K, tA, tB) in ((3016, 1448, 3656, 0, 0), (2200, 2432, 2400, 0, 1), (1184, 480, 2592, 0, 0),
                              (96, 3016, 3392, 1, 0), (768, 768, 3072, 0, 1)):
        A = torch.rand(M * K, device="cuda") * 2 - 1
        B = torch.rand(K * N, device="cuda") * 2 - 1
        C = torch.zeros(M * N, device="cuda")
        args = (tA, tB, M, N, K, 1.0, A, M if tA else K, B, K if tB else N, 0.0, C, N)
        ensure_workspace(ks, torch, 256 << 20)
        plan = ks.gemm_plan(ks.F32, -1, *args)
        kid = plan["kernel_id"]
        if plan["balanced_groups"] > 0:
            what = "balanced"
        elif plan["split_k"] > 1:
            what = "split_k"
        else:
            continue

        def timed():
            est = float(np.median(ks.time_gemm(ks.F32, kid, *args, warmup=1, iters=3, reps=1)))
            warm = int(min(64, max(2, np.ceil(30.0 / max(est, 1e-3)))))
            return float(np.median(ks.time_gemm(ks.F32, kid, *args, warmup=warm, iters=8, reps=1)))
        on = timed()
        if what == "balanced":
            ks.set_workspace(None)
            off = timed()
            ensure_workspace(ks, torch, 256 << 20)
        else:
            ks.set_split_partitions(1)
            off = timed()
            ks.set_split_partitions(0)
        fl = 2.0 * M * N * K
        out.append(dict(M=M, N=N, K=K, layout="NT"[tA] + "NT"[tB], form=what, kernel=kid, split_k=plan["split_k"],
                        balanced_groups=plan["balanced_groups"], ms=on, tflops=fl / (on * 1e-3) / 1e12,
                        ms_in_the_form_it_replaces=off, speedup=off / on))
        del A, B, C
    return out


def bf16_report(ks, torch):
    """Selected bf16 kernels on the large/skinny set: TFLOP/s, fraction of the bf16 matrix peak, and
    fraction of what a pure MFMA loop sustains on the same operand values in this run."""
    cells = time_set(ks, torch, "cfg5")
    g = torch.Generator(device="cuda")
    g.manual_seed(1000)
    ops = (torch.randn(ks.MFMA_PROBE_BYTES // 2, generator=g, device="cuda") / np.sqrt(8192.0)).to(torch.bfloat16)
    sustained, mhz = ks.mfma_sustained(ks.BF16, ops, rounds=4000)
    sustained16, mhz16 = ks.mfma_sustained(ks.BF16, ops, rounds=4000, fragment=16)
    zeros = torch.zeros(ks.MFMA_PROBE_BYTES // 2, dtype=torch.bfloat16, device="cuda")
    sustained0, mhz0 = ks.mfma_sustained(ks.BF16, zeros, rounds=4000)
    for c in cells:
        # against the pure loop of the fragment shape the cell's kernel uses
        f16 = ks.kernel_info(ks.BF16, c["kernel"])["core_name"] == "mfma16"
        c["frac_of_sustained_mfma"] = c["tflops"] / (sustained16 if f16 else sustained)
    big = [c for c in cells if min(c["M"], c["N"]) >= 2048]
    return dict(cells=cells, other_launch_forms=bf16_launch_forms(ks, torch),
                geomean_tflops=geomean([c["tflops"] for c in cells]),
                best_frac_of_peak=max(c["frac_of_peak"] for c in big),
                best_frac_of_sustained_mfma=max(c["frac_of_sustained_mfma"] for c in big),
                mfma_sustained=dict(what="ks_mfma_sustained: 2048 work-groups x 8 waves of 32x32x16 bf16 MFMAs on "
                                         "register operands, no LDS or memory traffic",
                                    normal_operands=dict(tflops=sustained, shader_mhz=mhz,
                                                         values="N(0,1)/sqrt(8192) rounded to bf16, as the cells use"),
                                    normal_operands_16x16x32=dict(tflops=sustained16, shader_mhz=mhz16),
                                    zero_operands=dict(tflops=sustained0, shader_mhz=mhz0)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg5", "fp32_large"])
    ap.add_argument("--single-launch", action="store_true", help="one launch per sample (profiler runs)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-extra", action="store_true", help="skip the reports measured after the timed region")
    ap.add_argument("--dump-rows", default=None, help="write per-row kernel id, time and TFLOP/s as CSV")
    a = ap.parse_args()
    if a.gpus != 1:
        raise SystemExit("bench.py measures one GPU: this build has no multi-GPU path; "
                         "run with --gpus 1")
    import torch
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs an MI355X (no CPU fallback exists)")
    import paper_2003_06795_amd.binding as ks

    # yardstick for hardware traffic counters: one plain copy of CALIB_BYTES, outside the timed region
    calib = torch.rand(2 * CALIB_BYTES // 4, device="cuda")
    ks.calibration_copy(calib[CALIB_BYTES // 4:], calib[:CALIB_BYTES // 4], CALIB_BYTES)
    torch.cuda.synchronize()
    del calib

    rows = build_rows(a.workload)
    dtype = rows[0]["dtype"]
    dt = ks.F32 if dtype == "f32" else ks.BF16
    bufs = allocate(rows, torch)
    workspace_for(ks, torch, rows)

    reps = reps_of(rows, a.single_launch)
    stream = torch.cuda.current_stream().cuda_stream
    probe = (torch.rand(ks.MFMA_PROBE_BYTES // 4, device="cuda") * 2 - 1) if dtype == "f32" else \
        torch.randn(ks.MFMA_PROBE_BYTES // 2, device="cuda").to(torch.bfloat16)
    for _ in range(a.warmup):
        run_pass(ks, rows, bufs, reps, stream)
    ms = np.zeros((a.steps, len(rows)))          # per-launch milliseconds, steps x rows
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(a.steps):
        run_pass(ks, rows, bufs, reps, stream, ms[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # the clock the device was left at by the pass (outside the timed region; see sustained_clock_report)
    mhz_after_pass = ks.mfma_sustained(dt, probe, rounds=20)[1]

    med = np.median(ms, axis=0)
    flops = flops_of(rows)
    tflops = flops / (med * 1e-3) / 1e12
    value = geomean(tflops)

    # what each row launched, from the library itself (same workspace as in the timed region)
    plans = [ks.gemm_plan(dt, -1, *gemm_args(r, bufs)) for r in rows]
    chosen = [p["kernel_id"] for p in plans]
    if a.dump_rows:
        with open(a.dump_rows, "w") as f:
            f.write("row,transA,transB,M,N,K,kernel,split_k,reps,median_ms,tflops\n")
            for i, r in enumerate(rows):
                f.write("%d,%d,%d,%d,%d,%d,%d,%d,%d,%.6g,%.6g\n" % (i, r["tA"], r["tB"], r["M"], r["N"], r["K"],
                                                                  chosen[i], plans[i]["split_k"], reps[i], med[i],
                                                                  tflops[i]))
    sym = [kernel_symbol(ks, dt, p, r["tA"], r["tB"]) for p, r in zip(plans, rows)]
    # Per kernel symbol: `pass_*` counts every row once (one pass of the workload = one GEMM per
    # row); `all_*` counts every timed launch (rows of few flops are repeated up to 64 times per
    # sample, a measurement device), which is what a profiler's per-symbol average sees.
    by = {}
    esz = 4 if dtype == "f32" else 2
    for i, s in enumerate(sym):
        # a row that runs more than one kernel inside its timed interval (split-K and its reduction,
        # a balanced launch that divides tiles and its second kernel, a hybrid launch) is booked
        # under a name of its own: its interval is not one kernel's duration
        multi = (plans[i]["split_k"] > 1 or plans[i]["tail_split"] > 0 or plans[i]["divided_tiles"] > 0 or
                 plans[i]["k_remainder"] > 0)
        d = by.setdefault(s + (" + further kernels" if multi else ""),
                          dict(pass_time=0.0, pass_flops=0.0, pass_bytes=0.0, rows=0, all_time=0.0, all_launches=0,
                               split=multi))
        r = rows[i]
        d["pass_time"] += float(med[i]) * 1e-3
        d["pass_flops"] += float(flops[i])
        d["pass_bytes"] += r["batch"] * ((r["M"] * r["K"] + r["K"] * r["N"]) * esz + r["M"] * r["N"] * 4)
        d["rows"] += 1
        d["all_time"] += float(ms[:, i].sum()) * 1e-3 * SAMPLES * reps[i]
        d["all_launches"] += a.steps * SAMPLES * reps[i]
    # The roofline is taken for the symbol that does the most flops in a pass among the rows that
    # run a single kernel (by flops and not by time, so that a run under a profiler, where the
    # microsecond rows are slowed to the host's enqueue rate, names the same kernel).
    single = [s_ for s_ in by if not by[s_]["split"]]
    dom = max(single or list(by), key=lambda s_: by[s_]["pass_flops"])
    d = by[dom]
    achieved = d["pass_flops"] / d["pass_time"] / 1e12
    traffic = stored_traffic(a.workload, dom)
    if traffic is not None:
        traffic["algorithmic_bytes"] = d["pass_bytes"] / d["rows"]
    pass_time = float(med.sum() * 1e-3)
    roofline = dict(bound="mfma", kernel=dom, achieved=achieved, peak=PEAK[dtype], unit="TFLOP/s",
                    frac=achieved / PEAK[dtype], traffic=traffic, launches_per_pass=d["rows"],
                    flops_per_launch=d["pass_flops"] / d["rows"],
                    avg_launch_us=d["pass_time"] / d["rows"] * 1e6,
                    avg_launch_us_over_all_timed_launches=d["all_time"] / d["all_launches"] * 1e6,
                    share_of_pass_time=d["pass_time"] / pass_time,
                    algorithmic_gbs=d["pass_bytes"] / d["pass_time"] / 1e9,
                    how=("achieved = flops_per_launch / avg_launch_us (HIP events, mean over the rows that "
                         "resolve to this symbol and run no other kernel in their timed interval)"))
    multi_rows = [v for v in by.values() if v["split"]]
    roofline["rows_with_more_than_one_kernel"] = dict(
        rows=int(sum(v["rows"] for v in multi_rows)),
        share_of_pass_time=float(sum(v["pass_time"] for v in multi_rows) / pass_time),
        what="split-K with its reduction, balanced launches that divide tiles, hybrid launches: not candidates")
    if multi_rows:
        # the largest of them, for the record: its interval is the sum of its kernels' durations
        name, v = max(((k, v) for k, v in by.items() if v["split"]), key=lambda kv: kv[1]["pass_time"])
        tf = v["pass_flops"] / v["pass_time"] / 1e12
        roofline["rows_with_more_than_one_kernel"]["largest"] = dict(
            kernels=name, rows=v["rows"], share_of_pass_time=v["pass_time"] / pass_time, tflops_over_the_interval=tf,
            frac_of_peak_over_the_interval=tf / PEAK[dtype], avg_interval_us=v["pass_time"] / v["rows"] * 1e6)

    out = {
        "metric": "GEMM TFLOP/s geomean over shape set; selected/exhaustive-best perf ratio",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": wall / a.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": {"cfg2": "fp32 tuning set: 200 log-uniform shapes in [16,4096]^3 (seed 1) x 4 layouts, "
                                        "selected kernel per row",
                                "cfg5": "bf16 large/skinny set: 7 shapes x {NN,NT}, selected kernel per row",
                                "fp32_large": "fp32 4096^3 in four layouts and three large im2col rows, selected kernel "
                                              "per row"}[a.workload],
                   "rows": len(rows), "kernels_used": len(set(chosen)),
                   "rows_that_split_k": int(sum(p["split_k"] > 1 for p in plans)),
                   "rows_with_a_split_last_round": int(sum(p["tail_split"] > 0 for p in plans)),
                   "rows_in_balanced_form": int(sum(p["balanced_groups"] > 0 for p in plans)),
                   "launches_per_step": int(sum(1 + SAMPLES * r for r in reps)),
                   "timing": ("per row and step: ks_time_gemm with 1 untimed launch and %d samples of `reps` back-to-back "
                              "launches between HIP events; row time = median over steps of the per-step median" % SAMPLES)},
        "timed_device_ms_per_step": float((ms * np.array(reps)[None, :]).sum() * SAMPLES / a.steps),
        "pass": dict(device_ms=pass_time * 1e3, tflops=float(flops.sum() / pass_time / 1e12),
                     frac_of_peak=float(flops.sum() / pass_time / 1e12 / PEAK[dtype]),
                     what="one GEMM per row: sum of flops / sum of per-launch times"),
        "best_row_tflops": float(tflops.max()),
        "frac_of_attainable": frac_summary(tflops, rows),
        "roofline": roofline,
    }
    # selector quality: stored (exhaustive sweep, held-out shapes) and live (this run)
    rep = os.path.join(ROOT, "paper_2003_06795_amd", "tune", "data", "tree_%s.json" % dtype)
    if os.path.exists(rep):
        R = json.load(open(rep))
        dep = [s for s in R["sweep"] if s["n_kept"] == R["deployed"]["n_kept"]][0]
        key = "2" if a.workload == "cfg2" else "6"
        held = dep.get("test_by_config", {}).get(key, dep["test"])
        out["selector"] = dict(source="stored exhaustive sweeps (%s), held-out 30%% of this workload's shapes"
                                      % ", ".join(os.path.basename(t) for t in R["timings"]),
                               leaf_limit=dep["n_kept"], kept=dep["kept"],
                               selected_over_best_geomean=held["selector"],
                               achievable_geomean=held["achievable"],
                               best_single_kernel_geomean=held["best_single"],
                               held_out_by_config={c: v["selector"] for c, v in dep.get("test_by_config", {}).items()})
    if not a.no_extra:
        sc = sustained_clock_report(ks, rows, bufs, reps, med, flops, dtype, probe, mhz_after_pass)
        if sc is not None:
            out["pass"]["at_sustained_clock"] = sc
    if not a.no_extra and a.workload == "cfg2":
        del bufs
        torch.cuda.empty_cache()
        out.setdefault("selector", {})["live"] = selector_live(ks, torch)
        large = time_set(ks, torch, "fp32_large")
        s32, mhz32 = ks.mfma_sustained(ks.F32, probe, rounds=2000)
        for c in large:
            c["frac_of_sustained_mfma"] = c["tflops"] / s32
        out["fp32_large"] = dict(cells=large, best_frac_of_peak=max(c["frac_of_peak"] for c in large),
                                 other_launch_forms=f32_launch_forms(ks, torch),
                                 mfma_sustained=dict(tflops=s32, shader_mhz=mhz32,
                                                     what="32x32x2 fp32 MFMAs on U[-1,1) register operands"))
        for name in ("cfg3_sample", "cfg4"):
            cells = time_set(ks, torch, name, iters=5)
            out[name] = dict(rows=len(cells), geomean_tflops=geomean([c["tflops"] for c in cells]),
                             frac_of_attainable_geomean=geomean([c["frac_of_attainable"] for c in cells]),
                             best=max(cells, key=lambda c: c["tflops"]))
        out["bf16_large"] = bf16_report(ks, torch)
        ks.set_workspace(None)
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
