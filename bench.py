#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg5]

A step is one pass of the deployed library over the workload: for every (shape, layout) row,
ks_select picks a kernel and ks_gemm_* runs it (inputs resident in HBM).  The default workload is
the fp32 tuning set (200 log-uniform shapes x 4 layouts = 800 GEMMs); `value` is the geometric
mean over rows of TFLOP/s, each row's time being the median over the K timed steps of the HIP
event interval around its launch.  One JSON line is printed with the roofline of the dominant
kernel and the CPU oracle timed on a bounded sample of the same rows.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"f32": 157.3, "bf16": 2516.6}      # dense matrix-core TFLOP/s of MI355X
HBM_TBS = 8.0                              # published HBM3E bandwidth, TB/s


def attainable_tflops(dtype, M, N, K, batch=1, beta=0.0):
    """Roofline bound of one GEMM: min(matrix peak, arithmetic intensity x HBM bandwidth), with the
    algorithmic bytes (each operand once, C written once and read once if beta != 0)."""
    esz = 4 if dtype == "f32" else 2
    by = batch * ((M * K + K * N) * esz + M * N * 4 * (2 if beta != 0.0 else 1))
    return min(PEAK[dtype], 2.0 * M * N * K * batch / by * HBM_TBS)
HBM_PEAK_GBS = 8000.0
CALIB_BYTES = 256 * 1024 * 1024
SAMPLES = 3                                 # timed samples per row per step


def kernel_symbol(ks, dt, kid, tA, tB, vec=True, dma=False):
    """Name of the device function a call resolves to (as rocprofv3 prints it).  dma: the bf16
    direct-to-LDS path applies (aligned operands and K a multiple of the K-step)."""
    ki = ks.kernel_info(dt, kid)
    akc, bkc = int(not tA), int(bool(tB))
    split = ki["split_k"] > 1
    b = lambda v: "true" if v else "false"
    if dt == ks.F32 and ki["core_name"] == "direct":
        return "gemm_f32_direct_kernel<%d, %d, %d, %d, %d, %s, %s, %s, %s>" % (
            ki["bm"], ki["bn"], ki["bk"], ki["wm"], ki["wn"], b(split), b(akc), b(bkc), b(vec))
    if dt == ks.F32 and ki["core_name"] == "kslice":
        return "gemm_f32_kslice_kernel<%d, %d, %d, %d, %d, %s, %s, %s, %s>" % (
            ki["bm"], ki["bn"], ki["bk"], ki["k_waves"], ki["wm"], b(split), b(akc), b(bkc), b(vec))
    if dt == ks.F32:
        p1, p2 = (ki["tm"], ki["tn"]) if ki["core_name"] == "fma" else (ki["wm"], ki["wn"])
        # last argument: the multi-tile form, which no row of the benchmark's workloads is large enough for
        return "gemm_f32_kernel<%d, %d, %d, %d, %d, %d, %s, %s, %s, %s, %d, false>" % (
            ki["core"], ki["bm"], ki["bn"], ki["bk"], p1, p2, b(split), b(akc), b(bkc), b(vec), ki["k_waves"])
    f = 16 if ki["core_name"] == "mfma16" else 32
    if vec and dma:
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
        C = torch.zeros(M * N * b, device="cuda")
        bufs[key] = (A, B, C)
    return bufs


def run_pass(ks, rows, bufs, reps, stream, out_ms=None):
    """One pass: every row's GEMM with the selected kernel (kernel id -1 = ks_select), timed the way
    the tuner times a cell (ks_time_gemm): one untimed launch, then SAMPLES samples of reps[i]
    back-to-back launches, each between one HIP event pair.  The untimed launch keeps the queue
    ahead of the device, so a sample measures kernel time and not the host's enqueue rate.
    out_ms[i] receives the median per-launch milliseconds of the samples."""
    for i, r in enumerate(rows):
        A, B, C = bufs[(r["dtype"], r["shape"])]
        M, N, K, b = r["M"], r["N"], r["K"], r["batch"]
        ms = ks.time_gemm(ks.F32 if r["dtype"] == "f32" else ks.BF16, -1, r["tA"], r["tB"], M, N, K,
                          r["alpha"], A, M if r["tA"] else K, B, K if r["tB"] else N, r["beta"], C, N, b,
                          M * K if b > 1 else 0, K * N if b > 1 else 0, M * N if b > 1 else 0,
                          stream=stream, warmup=1, iters=SAMPLES, reps=reps[i])
        if out_ms is not None:
            out_ms[i] = float(np.median(ms))


def stored_traffic(workload, symbol):
    """HBM bytes per launch of `symbol` from the committed counter summary (two rocprofv3 --pmc runs
    of this script, FETCH_SIZE and WRITE_SIZE, scaled by the calibration copy), or None."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic_%s.txt" % workload)
    if not os.path.exists(path):
        return None
    for k in json.load(open(path)).get("kernels", []):
        if k["kernel"] == symbol:
            return dict(fetch_bytes=k["fetch_bytes"], write_bytes=k["write_bytes"],
                        total_bytes=k["fetch_bytes"] + k["write_bytes"], algorithmic_bytes=k.get("algorithmic_bytes"))
    return None


def cpu_baseline(rows, budget_s=12.0):
    """The CPU oracle, as it stands, on a seeded sample of the same rows (small ones first so the
    sample is bounded); reports the geometric mean of its TFLOP/s over the sampled rows."""
    import workloads as wl
    from oracle import gemm as og
    order = np.random.default_rng(0).permutation(len(rows))
    picked, rates, spent = [], [], 0.0
    for i in order:
        r = rows[int(i)]
        macs = r["M"] * r["N"] * r["K"] * r["batch"]
        if macs > 2 ** 34 or spent > budget_s:
            continue
        p = wl.make_problem(r["dtype"], r["tA"], r["tB"], r["M"], r["N"], r["K"], batch=r["batch"],
                            alpha=r["alpha"], beta=r["beta"], seed=1, key=int(i),
                            dist="normal" if r["dtype"] == "bf16" else "uniform")
        C = p.C0.copy()
        t0 = time.perf_counter()
        og.gemm(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, C,
                p.ldc, p.batch, p.strideA, p.strideB, p.strideC)
        dt = time.perf_counter() - t0
        spent += dt
        picked.append(int(i))
        rates.append(2.0 * macs / dt / 1e12)
        if len(picked) >= 400:
            break
    return dict(value=float(np.exp(np.mean(np.log(rates)))), unit="TFLOP/s (geomean over sampled rows)",
                cores=og.num_threads(), kind="oracle",
                sample="%d seeded rows of the workload with M*N*K <= 2^34, full fp64 triple loop, %.1f s of CPU work"
                       % (len(picked), spent))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg5"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-extra", action="store_true", help="skip the bf16 large-shape report")
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
    need = max(ks.workspace_bytes_needed(dt, ks.select(dt, r["M"], r["N"], r["K"], r["batch"], r["tA"], r["tB"]),
                                         r["M"], r["N"], r["batch"]) for r in rows)
    ws = None
    if need:
        ws = torch.empty(need // 4 + 1, dtype=torch.float32, device="cuda")
        ks.set_workspace(ws)

    # Like the tuner, a row's sample is a short run of back-to-back launches (issued natively by
    # ks_time_gemm) so that the event interval measures kernel time rather than host dispatch.  The
    # repetition count is a fixed function of the row's flops (about 1.2e9 flops per sample, at
    # most 64 launches: roughly the tuner's 100 us samples), so warm-up and timed passes launch
    # exactly the same kernels.
    reps = [int(min(64, max(1, np.ceil(1.2e9 / (2.0 * r["M"] * r["N"] * r["K"] * r["batch"]))))) for r in rows]
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(a.warmup):
        run_pass(ks, rows, bufs, reps, stream)
    ms = np.zeros((a.steps, len(rows)))          # per-launch milliseconds, steps x rows
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(a.steps):
        run_pass(ks, rows, bufs, reps, stream, ms[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    med = np.median(ms, axis=0)
    flops = np.array([2.0 * r["M"] * r["N"] * r["K"] * r["batch"] for r in rows])
    tflops = flops / (med * 1e-3) / 1e12
    value = float(np.exp(np.mean(np.log(tflops))))

    # dominant kernel symbol: the instantiation with the most device time in a step
    chosen = [ks.select(dt, r["M"], r["N"], r["K"], r["batch"], r["tA"], r["tB"]) for r in rows]
    if a.dump_rows:
        with open(a.dump_rows, "w") as f:
            f.write("row,transA,transB,M,N,K,kernel,reps,median_ms,tflops\n")
            for i, r in enumerate(rows):
                f.write("%d,%d,%d,%d,%d,%d,%d,%d,%.6g,%.6g\n" % (i, r["tA"], r["tB"], r["M"], r["N"], r["K"],
                                                               chosen[i], reps[i], med[i], tflops[i]))
    sym = [kernel_symbol(ks, dt, k, r["tA"], r["tB"], vec=all(v % 8 == 0 for v in (r["M"], r["N"], r["K"])),
                         dma=dtype == "bf16" and r["K"] % ks.kernel_info(dt, k)["bk"] == 0)
           for k, r in zip(chosen, rows)]
    # Per kernel symbol: `pass_*` counts every row once (one pass of the workload = one GEMM per
    # row); `all_*` counts every timed launch (rows of few flops are repeated up to 64 times per
    # sample, a measurement device), which is what a profiler's per-symbol average sees.
    by = {}
    for i, s in enumerate(sym):
        d = by.setdefault(s, dict(pass_time=0.0, pass_flops=0.0, pass_bytes=0.0, rows=0, all_time=0.0,
                                  all_launches=0, split=ks.kernel_info(dt, chosen[i])["split_k"] > 1))
        r = rows[i]
        esz = 4 if dtype == "f32" else 2
        d["pass_time"] += float(med[i]) * 1e-3
        d["pass_flops"] += float(flops[i])
        d["pass_bytes"] += r["batch"] * ((r["M"] * r["K"] + r["K"] * r["N"]) * esz + r["M"] * r["N"] * 4)
        d["rows"] += 1
        d["all_time"] += float(ms[:, i].sum()) * 1e-3 * SAMPLES * reps[i]
        d["all_launches"] += a.steps * SAMPLES * reps[i]
    # A split-K GEMM is two kernels (partial products, then the fixed-order reduction) inside one
    # timed interval, so its interval is not one kernel's duration; the roofline is taken for the
    # symbol with the most time in a pass among the single-kernel GEMMs.
    single = [s_ for s_ in by if not by[s_]["split"]]
    dom = max(single or list(by), key=lambda s_: by[s_]["pass_time"])
    d = by[dom]
    achieved = d["pass_flops"] / d["pass_time"] / 1e12
    traffic = stored_traffic(a.workload, dom)
    if traffic is not None:
        traffic["algorithmic_bytes"] = d["pass_bytes"] / d["rows"]
    roofline = dict(bound="mfma", kernel=dom, achieved=achieved, peak=PEAK[dtype], unit="TFLOP/s",
                    frac=achieved / PEAK[dtype], traffic=traffic, launches_per_pass=d["rows"],
                    avg_launch_us=d["pass_time"] / d["rows"] * 1e6,
                    avg_launch_us_over_all_timed_launches=d["all_time"] / d["all_launches"] * 1e6,
                    share_of_pass_time=d["pass_time"] / float(med.sum() * 1e-3),
                    algorithmic_gbs=d["pass_bytes"] / d["pass_time"] / 1e9)

    out = {
        "metric": "GEMM TFLOP/s geomean over shape set; selected/exhaustive-best perf ratio",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": wall / a.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": ("fp32 tuning set: 200 log-uniform shapes in [16,4096]^3 (seed 1) x 4 layouts, "
                                "selected kernel per row" if a.workload == "cfg2" else
                                "bf16 large/skinny set: 7 shapes x {NN,NT}, selected kernel per row"),
                   "rows": len(rows), "kernels_used": len(set(chosen)),
                   "launches_per_step": int(sum(1 + SAMPLES * r for r in reps)),
                   "timing": ("per row and step: ks_time_gemm with 1 untimed launch and %d samples of `reps` back-to-back "
                              "launches between HIP events; row time = median over steps of the per-step median" % SAMPLES)},
        "timed_device_ms_per_step": float((ms * np.array(reps)[None, :]).sum() * SAMPLES / a.steps),
        "best_row_tflops": float(tflops.max()),
        "frac_of_attainable": frac_summary(tflops, rows),
        "roofline": roofline,
    }
    # selector quality measured offline on the stored exhaustive sweep (held-out shapes)
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
    if not a.no_extra and a.workload == "cfg2":
        out["bf16_large"] = bf16_report(ks, torch)
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(rows)
    print(json.dumps(out))


def frac_summary(tflops, rows):
    """Achieved / min(peak, AI x 8 TB/s) per row: geometric mean, quartiles and the maximum.  Most rows
    of the fp32 tuning set last a few microseconds, where launch latency (not in this bound) rules."""
    f = np.array([t / attainable_tflops(r["dtype"], r["M"], r["N"], r["K"], r["batch"])
                  for t, r in zip(tflops, rows)])
    q = np.quantile(f, [0.25, 0.5, 0.75])
    return dict(geomean=float(np.exp(np.mean(np.log(f)))), q25=float(q[0]), median=float(q[1]),
                q75=float(q[2]), max=float(f.max()))


def bf16_report(ks, torch):
    """Selected bf16 kernels on the large/skinny set: TFLOP/s and fraction of the bf16 matrix peak."""
    rows = build_rows("cfg5")
    bufs = allocate(rows, torch)
    ws = torch.empty(64 * 256 * 256 + 4 * 8192 * 256 + 1024, dtype=torch.float32, device="cuda")
    ks.set_workspace(ws)
    cells = []
    for r in rows:
        A, B, C = bufs[(r["dtype"], r["shape"])]
        M, N, K = r["M"], r["N"], r["K"]
        kid = ks.select(ks.BF16, M, N, K, 1, r["tA"], r["tB"])
        if ks.workspace_bytes_needed(ks.BF16, kid, M, N, 1) > ws.numel() * 4:
            continue
        t = ks.time_gemm(ks.BF16, kid, r["tA"], r["tB"], M, N, K, 1.0, A, M if r["tA"] else K, B,
                         K if r["tB"] else N, 0.0, C, N, warmup=3, iters=10, reps=1)
        tf = 2.0 * M * N * K / (float(np.median(t)) * 1e-3) / 1e12
        gbs = ((M * K + K * N) * 2 + M * N * 4) / (float(np.median(t)) * 1e-3) / 1e9
        cells.append(dict(M=M, N=N, K=K, layout="N" + "NT"[r["tB"]], kernel=kid, tflops=tf,
                          frac_of_bf16_peak=tf / PEAK["bf16"], algorithmic_gbs=gbs,
                          attainable_tflops=attainable_tflops("bf16", M, N, K),
                          frac_of_attainable=tf / attainable_tflops("bf16", M, N, K)))
    ks.set_workspace(None)
    big = [c["tflops"] for c in cells if min(c["M"], c["N"]) >= 2048]
    return dict(cells=cells, geomean_tflops=float(np.exp(np.mean(np.log([c["tflops"] for c in cells])))),
                best_frac_of_peak=max(big) / PEAK["bf16"] if big else None)


if __name__ == "__main__":
    main()
