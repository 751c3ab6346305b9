"""Shared plumbing of the GPU parity tests: seeded inputs -> oracle (CPU, fp64) and libsa (GPU)."""
import numpy as np
import torch

from oracle import binding as orc
from paper_2604_00754_amd import synth

# tolerances of the benchmark definition: bf16 max-abs 2e-2 and relative L2 5e-3; fp32 1e-5
TOL = {"bf16": (2e-2, 5e-3), "f32": (1e-5, 1e-5)}
# gradients are sums of O(W) bf16-rounded products; they are held to the same relative-L2 bar and
# to a max-abs bar scaled by the tensor's own magnitude
DEV = "cuda:0"


def tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_dev(x_f32: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(x_f32).to(DEV).to(tdtype(dtype)).contiguous()


def to_np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def errors(got: np.ndarray, ref: np.ndarray):
    diff = got.astype(np.float64) - ref
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))


def assert_close(got, ref, dtype, what, scale_abs=1.0):
    """max-abs and relative-L2 bars of the benchmark definition.  When the reference is (numerically)
    the zero tensor -- e.g. the gradient w.r.t. Q and K when every query sees a single key -- a
    relative error has no meaning and only the max-abs bar is applied."""
    ma, rl = errors(got, ref)
    amax, rmax = TOL[dtype]
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    ref_rms = float(np.sqrt(np.mean(ref.astype(np.float64) ** 2)))
    rel_ok = rl <= rmax or ref_rms < 1e-4
    assert ma <= amax * scale_abs and rel_ok, f"{what}: max-abs {ma:.3e} (<= {amax * scale_abs:.1e}) rel-L2 {rl:.3e} (<= {rmax:.1e})"
    return ma, rl


def make_case(B, Hq, Hkv, n, d, w, dtype="bf16", perm_B=1, perm_H=1, seed=0, gates=False, grads=False,
              identity=False):
    wl = synth.Workload("case", B, Hq, Hkv, n, d, w, dtype, perm_B=perm_B, perm_H=perm_H)
    need = ["Q", "K", "V"] + (["gate_sa", "gate_swa"] if gates else []) + (["dY"] if grads else [])
    x = synth.make_inputs(wl, seed=seed, need=need)
    x["perm"] = None if identity else synth.permutations(perm_B, perm_H, n, seed=seed)
    return wl, x


def orc_desc(wl, window, causal):
    return orc.desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, window, causal, wl.perm_B, wl.perm_H)


def sa_desc(wl, window, causal, gate_per_dim=0, gate_dtype=1):
    from paper_2604_00754_amd import binding as sa
    return sa.make_desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, window, causal,
                        sa.SA_BF16 if wl.dtype == "bf16" else sa.SA_F32, 0.0, wl.perm_B, wl.perm_H,
                        gate_per_dim, gate_dtype)


sample_rows = synth.sample_rows
