"""Seeded sweep of random shapes through sa_fwd and sa_bwd (bf16 and fp32) against the fp64 oracle: sizes that no
hand-picked case names — sequence lengths on and off tile edges, windows from 1 to beyond n, every window kind,
with and without the causal test, GQA ratios 1 to 8, shared / per-head / per-batch permutations and the identity."""
import numpy as np
import pytest

from tests.test_gpu_fwd import run_fwd
from tests.test_gpu_bwd import run_bwd

pytestmark = pytest.mark.gpu


def draw(g, dtype):
    Hkv = int(g.choice([1, 2, 3]))
    ratio = int(g.choice([1, 2, 4, 8] if dtype == "bf16" else [1, 2]))
    Hq = Hkv * ratio
    B = int(g.integers(1, 3))
    d = int(g.choice([64, 128]))
    n = int(g.choice([int(g.integers(1, 70)), int(g.integers(70, 700)), 32 * int(g.integers(1, 12)),
                      128 * int(g.integers(1, 5)) + int(g.integers(-1, 2))]))
    n = max(n, 1)
    if dtype == "f32":
        n = min(n, 300)
    w = int(g.choice([1, 2, int(g.integers(1, 2 * n + 3)), int(g.integers(1, 130)), n, n + 1]))
    window = int(g.integers(0, 3))
    causal = int(g.integers(0, 2))
    mode = int(g.integers(0, 4))          # 0 shared, 1 per head, 2 per batch and head, 3 identity
    perm_B, perm_H = (1, 1) if mode in (0, 3) else ((1, Hq) if mode == 1 else (B, Hq))
    return dict(B=B, Hq=Hq, Hkv=Hkv, n=n, d=d, w=w, window=window, causal=causal, dtype=dtype,
                perm_B=perm_B, perm_H=perm_H, identity=(mode == 3))


@pytest.mark.parametrize("dtype,count,seed", [("bf16", 24, 11), ("f32", 8, 12)])
def test_forward_random_shapes(dtype, count, seed):
    g = np.random.default_rng(seed)
    for k in range(count):
        run_fwd(seed=100 * seed + k, **draw(g, dtype))


@pytest.mark.parametrize("dtype,count,seed", [("bf16", 16, 21), ("f32", 6, 22)])
def test_backward_random_shapes(dtype, count, seed):
    g = np.random.default_rng(seed)
    for k in range(count):
        run_bwd(seed=100 * seed + k, **draw(g, dtype))
