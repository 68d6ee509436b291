"""Brute-force timing sweep (paper Section II-A): every kernel of the family on every workload.

    python -m paper_2003_06795_amd.tune.sweep --config 2 --out gpurun_out/timings_cfg2.csv

Each (workload, kernel) cell is timed inside the library (ks_time_gemm: HIP events around
back-to-back launches on the stream) with `--warmup` untimed launches and `--iters` samples whose
repetition count is chosen so a sample lasts at least `--min-sample-us`; the median per-launch
time is recorded.  Buffers are reused across launches (hot caches).  The CSV is append-only and
keyed by (config, row, kernel): re-running skips cells already present.
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
          "median_ms", "min_ms", "iters", "reps"]


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
    elif config == 7:
        for i, (s, tA, tB, M, N, K, b) in enumerate(wl.config2_extra_rows()):
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


def time_cell(dtype, kid, tA, tB, M, N, K, batch, alpha, beta, buf, warmup, iters, min_sample_us,
              max_cell_ms):
    lda, ldb, ldc = (M if tA else K), (K if tB else N), N
    sA, sB, sC = buf.strides
    args = (tA, tB, M, N, K, alpha, buf.A, lda, buf.B, ldb, beta, buf.C, ldc, batch, sA, sB, sC)
    dt = ks.F32 if dtype == "f32" else ks.BF16
    probe = float(ks.time_gemm(dt, kid, *args, warmup=1, iters=1, reps=1)[0])
    reps = int(min(256, max(1, np.ceil(min_sample_us * 1e-3 / max(probe, 1e-4)))))
    n = int(max(3, min(iters, max_cell_ms / max(probe * reps, 1e-4))))
    w = int(max(0, min(warmup, max_cell_ms / max(probe, 1e-4) / 4)))
    ms = ks.time_gemm(dt, kid, *args, warmup=w, iters=n, reps=reps)
    return float(np.median(ms)), float(np.min(ms)), n, reps


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True)
    ap.add_argument("--out", required=True)
    ap.add_argument("--limit", type=int, default=None, help="config 3: size of the seeded subsample")
    ap.add_argument("--kernels", default=None, help="comma list of kernel ids (default: all)")
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
    if os.path.exists(a.out):
        with open(a.out) as f:
            for r in csv.DictReader(f):
                done.add((int(r["config"]), int(r["row"]), int(r["kernel"])))
    os.makedirs(os.path.dirname(os.path.abspath(a.out)), exist_ok=True)
    new = not os.path.exists(a.out)
    out = open(a.out, "a", newline="")
    wr = csv.DictWriter(out, FIELDS)
    if new:
        wr.writeheader()
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
            med, mn, n, reps = time_cell(dtype, kid, tA, tB, M, N, K, batch, alpha, beta, buf,
                                         a.warmup, a.iters, a.min_sample_us, a.max_cell_ms)
            wr.writerow(dict(config=a.config, row=ri, dtype=dtype, transA=tA, transB=tB, M=M, N=N, K=K,
                             batch=batch, kernel=kid, median_ms="%.6g" % med, min_ms="%.6g" % mn,
                             iters=n, reps=reps))
        out.flush()
        del buf
        if time.time() - last > 20:
            last = time.time()
            print("[sweep] config %d: %d / %d rows, %.0f s" % (a.config, n_row + 1, len(rows), last - t0),
                  flush=True)
    out.close()
    print("[sweep] done: %d rows in %.0f s -> %s" % (len(rows), time.time() - t0, a.out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
