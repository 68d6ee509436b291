"""Brute-force timing sweep (paper Section II-A): every kernel of the family on every workload.

    python -m paper_2003_06795_amd.tune.sweep --config 2 --out timings_cfg2.csv

Each (workload, kernel) cell is timed inside the library (ks_time_gemm: HIP events around
back-to-back launches on the stream) with `--warmup` untimed launches and `--iters` samples whose
repetition count is chosen so a sample lasts at least `--min-sample-us`; the median per-launch
time is recorded.  Buffers are reused across launches (hot caches).  The CSV is append-only and
keyed by (config, row, kernel): re-running skips cells already present; `--retime` with `--kernels`
drops the stored cells of those kernels first (after a kernel's code has changed).

Before a cell is timed its first launch is checked: sampled entries of its output must agree with
those of the row's reference member (the first kernel of the family that needs no workspace, whose
own results the parity tests pin) within twice the stated accuracy bound.  A cell that fails is
recorded as unusable (1e9 ms, check = fail), so a kernel that computes something else can never win
a row of the table.
"""
import argparse
import csv
import os
import sys
import time

import numpy as np
import torch

import workloads as wl
from .. import binding as ks

FIELDS = ["config", "row", "dtype", "transA", "transB", "M", "N", "K", "batch", "kernel",
          "median_ms", "min_ms", "iters", "reps", "check"]
REFERENCE_KERNEL = {"f32": 22, "bf16": 5}       # LDS-staged MFMA members without split-K
CHECK_SAMPLES = 4096


def rows_of(config, limit=None, seed=0):
    """[(row_index, dtype, tA, tB, M, N, K, batch, alpha, beta)]"""
    out = []
    if config == 2:
        for i, (s, tA, tB, M, N, K, b) in enumerate(wl.config2_rows()):
            out.append((i, "f32", tA, tB, M, N, K, b, 1.0, 0.0))
    elif config == 3:
        shapes = wl.config3_shapes()
        idx = np.arange(len(shapes))
        if limit is not None and limit < len(shapes):
            idx = np.sort(np.random.default_rng([3, seed]).choice(len(shapes), limit, replace=False))
        for i in idx:
            M, N, K = shapes[int(i)]
            out.append((int(i), "f32", 0, 0, M, N, K, 1, 1.0, 0.0))
    elif config == 4:
        for i, (M, N, K) in enumerate(wl.config4_shapes()):
            out.append((i, "f32", 0, 0, M, N, K, wl.CONFIG4_BATCH, wl.CONFIG4_ALPHA, wl.CONFIG4_BETA))
    elif config == 5:
        i = 0
        for (M, N, K) in wl.config5_shapes():
            for (tA, tB) in wl.CONFIG5_LAYOUTS:
                out.append((i, "bf16", tA, tB, M, N, K, 1, 1.0, 0.0))
                i += 1
    elif config == 8:
        # more rows of the bf16 tuning distribution (other seed): training only
        i = 0
        for (M, N, K) in wl.bf16_tuning_shapes(n=320, seed=15):
            for (tA, tB) in wl.CONFIG5_LAYOUTS:
                out.append((i, "bf16", tA, tB, M, N, K, 1, 1.0, 0.0))
                i += 1
    elif config == 9:
        # the bf16 tuning shapes (config 6) with A stored K x M: layouts TN and TT
        i = 0
        for (M, N, K) in wl.bf16_tuning_shapes():
            for (tA, tB) in ((1, 0), (1, 1)):
                out.append((i, "bf16", tA, tB, M, N, K, 1, 1.0, 0.0))
                i += 1
    elif config == 7:
        for i, (s, tA, tB, M, N, K, b) in enumerate(wl.config2_extra_rows()):
            out.append((i, "f32", tA, tB, M, N, K, b, 1.0, 0.0))
    elif config == 12:
        # large fp32 shapes (all three dimensions 2048 .. 8192): training only
        for i, (s, tA, tB, M, N, K, b) in enumerate(wl.large_fp32_rows()):
            out.append((i, "f32", tA, tB, M, N, K, b, 1.0, 0.0))
    elif config == 13:
        # medium-to-large fp32 shapes (dimensions 1024 .. 8192): training only
        for i, (s, tA, tB, M, N, K, b) in enumerate(wl.medium_large_fp32_rows()):
            out.append((i, "f32", tA, tB, M, N, K, b, 1.0, 0.0))
    elif config == 11:
        # more batched small shapes (other dimensions and batch sizes): training only
        for i, (M, N, K, b) in enumerate(wl.config4_extra_rows()):
            out.append((i, "f32", 0, 0, M, N, K, b, wl.CONFIG4_ALPHA, wl.CONFIG4_BETA))
    elif config == 6:
        i = 0
        for (M, N, K) in wl.bf16_tuning_shapes():
            for (tA, tB) in wl.CONFIG5_LAYOUTS:
                out.append((i, "bf16", tA, tB, M, N, K, 1, 1.0, 0.0))
                i += 1
    else:
        raise ValueError(config)
    return out


class Buffers:
    """Device operands for one workload: seeded uniform[-1,1) (normal/sqrt(K) for bf16), dense."""

    def __init__(self, dtype, M, N, K, batch, seed):
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        nA, nB, nC = M * K * batch, K * N * batch, M * N * batch
        if dtype == "f32":
            self.A = torch.rand(nA, generator=g, device="cuda") * 2 - 1
            self.B = torch.rand(nB, generator=g, device="cuda") * 2 - 1
        else:
            s = 1.0 / np.sqrt(max(K, 1))
            self.A = (torch.randn(nA, generator=g, device="cuda") * s).to(torch.bfloat16)
            self.B = (torch.randn(nB, generator=g, device="cuda") * s).to(torch.bfloat16)
        self.C = torch.rand(nC, generator=g, device="cuda") * 2 - 1
        self.strides = (M * K, K * N, M * N) if batch > 1 else (0, 0, 0)


class Checker:
    """First-launch check of a row: the reference member's output on sampled entries."""

    def __init__(self, dtype, tA, tB, M, N, K, batch, alpha, beta, buf):
        self.dt = ks.F32 if dtype == "f32" else ks.BF16
        lda, ldb = (M if tA else K), (K if tB else N)
        sA, sB, sC = buf.strides
        self.head = (tA, tB, M, N, K, alpha, buf.A, lda, buf.B, ldb, beta)
        self.tail = (N, batch, sA, sB, sC)
        self.C0 = buf.C.clone()
        n = buf.C.numel()
        g = torch.Generator(device="cuda")
        g.manual_seed(12345)
        self.idx = torch.randint(0, n, (min(CHECK_SAMPLES, n),), generator=g, device="cuda")
        self.idx[0], self.idx[-1] = 0, n - 1
        self.scratch = torch.empty_like(buf.C)
        self.ref = self.sample(REFERENCE_KERNEL[dtype])
        # twice the stated bound (both sides carry it), values drawn from [-1, 1) or N(0,1)/sqrt(K)
        amax = float(buf.A.abs().max()) * float(buf.B.abs().max())
        rel = 1e-5 * K if dtype == "f32" else 1e-2 * np.sqrt(max(K, 1))
        self.tol = 2.0 * (abs(alpha) * rel * amax + 1e-6 * abs(beta) * float(self.C0.abs().max())) + 1e-30

    def sample(self, kid):
        self.scratch.copy_(self.C0)
        fn = ks.gemm_f32_with_kernel if self.dt == ks.F32 else ks.gemm_bf16_with_kernel
        fn(kid, *self.head, self.scratch, *self.tail)
        return self.scratch[self.idx].clone()

    def ok(self, kid):
        got = self.sample(kid)
        err = float((got - self.ref).abs().max())
        return bool(torch.isfinite(got).all()) and err <= self.tol


HEAVY_MS = 0.02          # cells of at least 20 us per launch are taken at the sustained clock
HEAT_MS = 30.0           # load that brings the shader clock from its idle level to the sustained one
_last_heavy = [-1e9]     # perf_counter() at the end of the last heavy cell


def time_cell(dtype, kid, tA, tB, M, N, K, batch, alpha, beta, buf, warmup, iters, min_sample_us,
              max_cell_ms):
    """Median and minimum per-launch milliseconds of one (kernel, problem) cell.

    The shader clock follows the load: after idle, a buffer fill or a stretch of microsecond
    kernels it sits 10 - 15 % below the clock it reaches after 25 - 30 ms of dense work.  A sweep
    over all members keeps the device at the sustained clock by itself (64 kernels in a row on one
    shape), a sweep over a few members (--kernels) does not, and its cells would read slower than
    the stored ones they are compared with.  So a heavy cell that does not follow another heavy
    cell within a few milliseconds is preceded by HEAT_MS of its own launches."""
    lda, ldb, ldc = (M if tA else K), (K if tB else N), N
    sA, sB, sC = buf.strides
    args = (tA, tB, M, N, K, alpha, buf.A, lda, buf.B, ldb, beta, buf.C, ldc, batch, sA, sB, sC)
    dt = ks.F32 if dtype == "f32" else ks.BF16
    probe = float(ks.time_gemm(dt, kid, *args, warmup=1, iters=1, reps=1)[0])
    heavy = probe >= HEAVY_MS
    if heavy and time.perf_counter() - _last_heavy[0] > 0.005:
        ks.time_gemm(dt, kid, *args, warmup=int(min(2000, np.ceil(HEAT_MS / probe))), iters=1, reps=1)
    reps = int(min(256, max(1, np.ceil(min_sample_us * 1e-3 / max(probe, 1e-4)))))
    n = int(max(3, min(iters, max_cell_ms / max(probe * reps, 1e-4))))
    w = int(max(0, min(warmup, max_cell_ms / max(probe, 1e-4) / 4)))
    ms = ks.time_gemm(dt, kid, *args, warmup=w, iters=n, reps=reps)
    if heavy:
        _last_heavy[0] = time.perf_counter()
    return float(np.median(ms)), float(np.min(ms)), n, reps


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True)
    ap.add_argument("--out", required=True)
    ap.add_argument("--limit", type=int, default=None, help="config 3: size of the seeded subsample")
    ap.add_argument("--kernels", default=None, help="comma list of kernel ids (default: all)")
    ap.add_argument("--retime", action="store_true",
                    help="with --kernels: drop the stored cells of those kernels of this config and time them again")
    ap.add_argument("--no-check", action="store_true", help="skip the first-launch check of every cell")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--min-sample-us", type=float, default=100.0)
    ap.add_argument("--max-cell-ms", type=float, default=400.0)
    ap.add_argument("--max-workspace-gib", type=float, default=2.0,
                    help="split-K cells needing more scratch than this are recorded as unusable")
    ap.add_argument("--max-elems", type=float, default=6e9, help="skip workloads with more operand elements")
    a = ap.parse_args(argv)

    rows = rows_of(a.config, a.limit)
    done = set()
    fields = FIELDS
    if os.path.exists(a.out):
        with open(a.out) as f:
            rd = csv.DictReader(f)
            fields = rd.fieldnames or FIELDS           # an older table without the check column keeps its layout
            kept = list(rd)
        if a.retime and a.kernels:
            drop = {int(k) for k in a.kernels.split(",")}
            kept = [r for r in kept if not (int(r["config"]) == a.config and int(r["kernel"]) in drop)]
            tmp = a.out + ".tmp"
            with open(tmp, "w", newline="") as f:
                w = csv.DictWriter(f, fields)
                w.writeheader()
                w.writerows(kept)
            os.replace(tmp, a.out)
        for r in kept:
            done.add((int(r["config"]), int(r["row"]), int(r["kernel"])))
    os.makedirs(os.path.dirname(os.path.abspath(a.out)), exist_ok=True)
    new = not os.path.exists(a.out)
    out = open(a.out, "a", newline="")
    wr = csv.DictWriter(out, fields, extrasaction="ignore")
    if new:
        wr.writeheader()
    failed = 0
    ws = None
    t0 = time.time()
    last = t0
    for n_row, (ri, dtype, tA, tB, M, N, K, batch, alpha, beta) in enumerate(rows):
        dt = ks.F32 if dtype == "f32" else ks.BF16
        kids = ([int(k) for k in a.kernels.split(",")] if a.kernels else list(range(ks.num_kernels(dt))))
        kids = [k for k in kids if (a.config, ri, k) not in done]
        if not kids:
            continue
        if (M * K + K * N + M * N) * batch > a.max_elems:
            print("[sweep] skip row %d (%d x %d x %d): too large" % (ri, M, N, K), flush=True)
            continue
        buf = Buffers(dtype, M, N, K, batch, seed=1000 * a.config + ri)
        chk = None if a.no_check else Checker(dtype, tA, tB, M, N, K, batch, alpha, beta, buf)
        for kid in kids:
            need = ks.workspace_bytes_needed(dt, kid, M, N, batch)
            if need > a.max_workspace_gib * 2 ** 30:
                # the split-K form is not usable here: recorded as (practically) infinitely slow
                wr.writerow(dict(config=a.config, row=ri, dtype=dtype, transA=tA, transB=tB, M=M, N=N, K=K,
                                 batch=batch, kernel=kid, median_ms="1e9", min_ms="1e9", iters=0, reps=0))
                continue
            if need and (ws is None or ws.numel() * 4 < need):
                ks.set_workspace(None)
                ws = None
                ws = torch.empty(need // 4 + 1, dtype=torch.float32, device="cuda")
                ks.set_workspace(ws)
            if chk is not None and not chk.ok(kid):
                failed += 1
                print("[sweep] CHECK FAILED config %d row %d kernel %d (%d x %d x %d, %d%d): recorded unusable"
                      % (a.config, ri, kid, M, N, K, tA, tB), flush=True)
                wr.writerow(dict(config=a.config, row=ri, dtype=dtype, transA=tA, transB=tB, M=M, N=N, K=K,
                                 batch=batch, kernel=kid, median_ms="1e9", min_ms="1e9", iters=0, reps=0,
                                 check="fail"))
                continue
            med, mn, n, reps = time_cell(dtype, kid, tA, tB, M, N, K, batch, alpha, beta, buf,
                                         a.warmup, a.iters, a.min_sample_us, a.max_cell_ms)
            wr.writerow(dict(config=a.config, row=ri, dtype=dtype, transA=tA, transB=tB, M=M, N=N, K=K,
                             batch=batch, kernel=kid, median_ms="%.6g" % med, min_ms="%.6g" % mn,
                             iters=n, reps=reps, check="ok" if chk is not None else ""))
        out.flush()
        del buf, chk
        if time.time() - last > 20:
            last = time.time()
            print("[sweep] config %d: %d / %d rows, %.0f s" % (a.config, n_row + 1, len(rows), last - t0),
                  flush=True)
    out.close()
    print("[sweep] done: %d rows in %.0f s -> %s; cells that failed the check: %d"
          % (len(rows), time.time() - t0, a.out, failed), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
