"""CPU oracle for the bf16 GEMM + fused-epilogue path.  Test infrastructure only.

Nothing in the product package may import this; only tests, the smoke check and
the benchmark's cpu_baseline leg do.
"""
