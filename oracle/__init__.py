"""fp64 CPU oracle for Stochastic Attention -- test infrastructure only.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this.
"""
