"""What bounds the large bf16 GEMM on this device, measured on the benchmark's own operand values:

    python -m paper_2003_06795_amd.tune.ceiling [--size 8192] > profiles/gemm_bf16_ceiling.txt

* the matrix pipe alone (ks_mfma_sustained): a pure MFMA loop on register operands, on zeros and
  on N(0,1)/sqrt(K) values; the clock the device holds, and with it the rate, depends on the values;
* the two-group 256 x 256 x 64 kernel with its data paths left out one at a time
  (ks_bf16_ablation): what the global -> LDS path and the LDS -> register path cost;
* the kernel itself through ks_gemm_bf16_with_kernel.
"""
import argparse
import json

import numpy as np
import torch

from .. import binding as ks

PEAK = 2516.6


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--size", type=int, default=8192)
    ap.add_argument("--iters", type=int, default=20)
    a = ap.parse_args()
    n = a.size
    g = torch.Generator(device="cuda")
    g.manual_seed(1234)
    A = (torch.randn(n * n, generator=g, device="cuda") / np.sqrt(n)).to(torch.bfloat16)
    B = (torch.randn(n * n, generator=g, device="cuda") / np.sqrt(n)).to(torch.bfloat16)
    C = torch.zeros(n * n, device="cuda")
    Z = torch.zeros(n * n, dtype=torch.bfloat16, device="cuda")
    flops = 2.0 * n ** 3
    out = dict(what="bf16 %d^3 NT, operands N(0,1)/sqrt(K) unless stated; TFLOP/s; published dense bf16 peak %.1f" % (n, PEAK))
    tf0, mhz0 = ks.mfma_sustained(ks.BF16, Z, rounds=4000)
    tf1, mhz1 = ks.mfma_sustained(ks.BF16, A, rounds=4000)
    out["mfma_only"] = dict(zero_operands=dict(tflops=tf0, shader_mhz=mhz0, frac_of_peak=tf0 / PEAK),
                            normal_operands=dict(tflops=tf1, shader_mhz=mhz1, frac_of_peak=tf1 / PEAK))
    names = {0: "full kernel", 1: "no global -> LDS loads", 2: "no LDS -> register reads", 3: "neither (MFMAs, barriers, C write)"}
    out["kernel_with_paths_left_out"] = {}
    for operands, (X, Y) in (("normal_operands", (A, B)), ("zero_operands", (Z, Z))):
        for mode in (0, 1, 2, 3):
            ms = float(np.median(ks.bf16_ablation(mode, X, Y, C, n, n, n, iters=a.iters)))
            out["kernel_with_paths_left_out"].setdefault(operands, {})[names[mode]] = dict(
                ms=ms, tflops=flops / ms / 1e9, frac_of_peak=flops / ms / 1e9 / PEAK,
                frac_of_mfma_only=flops / ms / 1e9 / (tf1 if operands == "normal_operands" else tf0))
    t = ks.time_gemm(ks.BF16, 2, 0, 1, n, n, n, 1.0, A, n, B, n, 0.0, C, n, warmup=3, iters=a.iters, reps=1)
    ms = float(np.median(t))
    out["ks_gemm_bf16_with_kernel_2"] = dict(ms=ms, tflops=flops / ms / 1e9, frac_of_peak=flops / ms / 1e9 / PEAK,
                                             frac_of_mfma_only=flops / ms / 1e9 / tf1)
    print(json.dumps(out, indent=1))


if __name__ == "__main__":
    main()
