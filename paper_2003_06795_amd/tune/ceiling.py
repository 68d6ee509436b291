"""What bounds the large bf16 GEMM on this device, measured on the benchmark's own operand values:

    python -m paper_2003_06795_amd.tune.ceiling [--size 8192] > profiles/gemm_bf16_ceiling.txt

* the matrix pipe alone (ks_mfma_sustained): a pure MFMA loop on register operands, on zeros and
  on N(0,1)/sqrt(K) values; the clock the device holds, and with it the rate, depends on the values;
* the two-group 256 x 256 x 64 kernel with its data paths left out one at a time
  (ks_bf16_ablation): what the global -> LDS path and the LDS -> register path cost;
* the clock the device holds while the whole kernel runs (work-group 0 reads the cycle and reference
  counters around its K loop), and the kernel's rate against the matrix pipe alone at that clock;
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
    tf16, mhz16 = ks.mfma_sustained(ks.BF16, A, rounds=4000, fragment=16)
    out["mfma_only"] = dict(zero_operands=dict(tflops=tf0, shader_mhz=mhz0, frac_of_peak=tf0 / PEAK),
                            normal_operands=dict(tflops=tf1, shader_mhz=mhz1, frac_of_peak=tf1 / PEAK),
                            normal_operands_16x16x32=dict(tflops=tf16, shader_mhz=mhz16, frac_of_peak=tf16 / PEAK))
    names = {0: "full kernel", 1: "no global -> LDS loads", 2: "no LDS -> register reads", 3: "neither (MFMAs, barriers, C write)"}
    out["kernel_with_paths_left_out"] = {}
    for operands, (X, Y) in (("normal_operands", (A, B)), ("zero_operands", (Z, Z))):
        for mode in (0, 1, 2, 3):
            ms = float(np.median(ks.bf16_ablation(mode, X, Y, C, n, n, n, iters=a.iters)))
            out["kernel_with_paths_left_out"].setdefault(operands, {})[names[mode]] = dict(
                ms=ms, tflops=flops / ms / 1e9, frac_of_peak=flops / ms / 1e9 / PEAK,
                frac_of_mfma_only=flops / ms / 1e9 / (tf1 if operands == "normal_operands" else tf0))
    # the clock the device holds while the whole kernel runs, and the kernel against what the matrix
    # pipe alone would do at THAT clock (the pure MFMA loop scaled by the ratio of the clocks)
    out["kernel_clock"] = {}
    for operands, mode, (X, Y), (tf_only, mhz_only) in (("normal_operands", 4, (A, B), (tf1, mhz1)),
                                                        ("normal_operands_16x16x32", 5, (A, B), (tf16, mhz16)),
                                                        ("normal_operands_16x16x32_all_loads_hit_L2", 6, (A, B), (tf16, mhz16)),
                                                        ("zero_operands", 4, (Z, Z), (tf0, mhz0))):
        ms4, mhz = ks.bf16_ablation(mode, X, Y, C, n, n, n, iters=a.iters)
        ms4 = float(np.median(ms4))
        tf = flops / ms4 / 1e9
        out["kernel_clock"][operands] = dict(ms=ms4, tflops=tf, shader_mhz=mhz, mfma_only_shader_mhz=mhz_only,
                                             mfma_only_tflops_at_kernel_clock=tf_only * mhz / mhz_only,
                                             frac_of_mfma_only_at_kernel_clock=tf / (tf_only * mhz / mhz_only))
    t = ks.time_gemm(ks.BF16, 2, 0, 1, n, n, n, 1.0, A, n, B, n, 0.0, C, n, warmup=3, iters=a.iters, reps=1)
    ms = float(np.median(t))
    out["ks_gemm_bf16_with_kernel_2"] = dict(ms=ms, tflops=flops / ms / 1e9, frac_of_peak=flops / ms / 1e9 / PEAK,
                                             frac_of_mfma_only=flops / ms / 1e9 / tf1)
    t = ks.time_gemm(ks.BF16, 44, 0, 1, n, n, n, 1.0, A, n, B, n, 0.0, C, n, warmup=3, iters=a.iters, reps=1)
    ms = float(np.median(t))
    out["ks_gemm_bf16_with_kernel_44_16x16x32"] = dict(ms=ms, tflops=flops / ms / 1e9, frac_of_peak=flops / ms / 1e9 / PEAK,
                                                       frac_of_mfma_only=flops / ms / 1e9 / tf16)
    print(json.dumps(out, indent=1))


if __name__ == "__main__":
    main()
