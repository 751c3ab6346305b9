"""Stochastic Attention hot path for AMD MI355X (gfx950): hand-written HIP kernels behind a C ABI."""
