"""CPU oracle: test infrastructure only.

Plain, slow, obviously-correct implementations of what the GPU path computes
(the GEMM of Section II and the prune/select pipeline of Sections III-IV of the
paper).  Only tests, the smoke check and the CPU-baseline leg of the benchmark
may import this package; the product package never does, and this package never
imports the product package.
"""
