"""Seeded synthetic inputs shaped like the paper's workloads.

Holds NONE of the method's arithmetic: only random tensors, random permutations
and the table of workload shapes.  Both the HIP path's tests/bench and the CPU
oracle's tests draw their inputs from here, so the two sides see identical data.

Values: Q, K, V, dY and gate logits are i.i.d. N(0,1) (numpy PCG64, one stream
per tensor); permutations are uniform over S_n (numpy's Fisher-Yates shuffle),
one per (batch, head) slice asked for.  Window/mask fields follow the paper:
the stochastic branch uses the circular symmetric window in permuted space and
the causal constraint on original positions (App. B mask); the sliding-window
branch uses the one-sided causal window (Sec. 3.1 footnote).
"""
from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 20260400754
_SLOT = {"Q": 0, "K": 1, "V": 2, "dY": 3, "gate_sa": 4, "gate_swa": 5}

WIN_SYM_CIRCULAR, WIN_SYM_LINEAR, WIN_ONE_SIDED = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    n: int
    d: int
    w: int
    dtype: str            # "bf16" | "f32"
    perm_B: int = 1
    perm_H: int = 1       # 1: one permutation per layer shared by heads; Hq: one per head
    gated: bool = False
    backward: bool = False

    def scaled(self, **kw):
        return replace(self, **kw)


# The five configurations the benchmark definition lists (index = position there).
WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", 1, 2, 2, 1024, 64, 64, "f32", perm_H=2),
    "pretrain_gated_2k": Workload("pretrain_gated_2k", 8, 12, 12, 2048, 64, 128, "bf16",
                                  perm_H=12, gated=True),
    "qwen3_8b_prefill_32k": Workload("qwen3_8b_prefill_32k", 1, 32, 8, 32768, 128, 512, "bf16"),
    "pretrain_fwdbwd_8k": Workload("pretrain_fwdbwd_8k", 4, 16, 16, 8192, 64, 256, "bf16",
                                   gated=True, backward=True),
    "qwen3_30b_prefill_128k": Workload("qwen3_30b_prefill_128k", 1, 32, 4, 131072, 128, 1024,
                                       "bf16"),
}


def _rng(seed_offset: int, layer: int = 0):
    return np.random.Generator(np.random.PCG64([BASE_SEED, seed_offset, layer]))


def normal(shape, which: str, layer: int = 0, seed: int = 0) -> np.ndarray:
    """float32 N(0,1) tensor; `which` picks the per-tensor stream."""
    return _rng(_SLOT[which] + 16 * seed, layer).standard_normal(shape, dtype=np.float32)


def permutations(perm_B: int, perm_H: int, n: int, layer: int = 0, seed: int = 0) -> np.ndarray:
    """int32 [perm_B, perm_H, n]; slice (b,h) is an independent uniform permutation whose
    entry p is the original index of the token placed at slot p."""
    out = np.empty((perm_B, perm_H, n), np.int32)
    for b in range(perm_B):
        for h in range(perm_H):
            g = np.random.Generator(np.random.PCG64([BASE_SEED, 1000 + seed, layer, b, h]))
            out[b, h] = g.permutation(n).astype(np.int32)
    return out


def identity_permutations(perm_B: int, perm_H: int, n: int) -> np.ndarray:
    return np.broadcast_to(np.arange(n, dtype=np.int32), (perm_B, perm_H, n)).copy()


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


def make_inputs(wl: Workload, layer: int = 0, seed: int = 0, need=("Q", "K", "V")):
    """dict of float32 arrays already rounded to the workload's storage dtype."""
    shapes = {"Q": (wl.B, wl.Hq, wl.n, wl.d), "K": (wl.B, wl.Hkv, wl.n, wl.d),
              "V": (wl.B, wl.Hkv, wl.n, wl.d), "dY": (wl.B, wl.Hq, wl.n, wl.d),
              "gate_sa": (wl.B, wl.Hq, wl.n), "gate_swa": (wl.B, wl.Hq, wl.n)}
    out = {}
    for k in need:
        x = normal(shapes[k], k, layer, seed)
        if wl.dtype == "bf16" and not k.startswith("gate"):
            x = round_to_bf16(x)
        out[k] = x
    return out


def sample_rows(B: int, H: int, n: int, per_head: int, seed: int) -> np.ndarray:
    """int32 [B*H*min(per_head,n), 3] of (b, h, i): a seeded sample of rows, every head covered."""
    g = np.random.Generator(np.random.PCG64([BASE_SEED, 2000 + seed]))
    m = min(per_head, n)
    out = np.empty((B, H, m, 3), np.int32)
    for b in range(B):
        for h in range(H):
            out[b, h, :, 0] = b
            out[b, h, :, 1] = h
            out[b, h, :, 2] = np.arange(n) if m == n else np.sort(g.choice(n, size=m, replace=False))
    return out.reshape(-1, 3)
