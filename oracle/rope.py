"""Oracle of rotary position embeddings on ORIGINAL token positions (test infrastructure only; numpy,
fp64, no code shared with the HIP library).

App. B (architecture, "Attention" item), App. C (training setup) and Sec. 4.2: RoPE (Su et al. 2023) is
applied to Q and K with each token's original sequence position, before any shuffling; the
permutation therefore never enters this operation.  RoFormer, Sec. 3.2.2: feature pair number i of a
row at position m is rotated by the angle m * theta_i, theta_i = base^(-2 i / d), i = 0 .. d/2 - 1:

    (a, b) -> (a cos(m theta_i) - b sin(m theta_i),  a sin(m theta_i) + b cos(m theta_i))

Which two features form pair i is not fixed by the paper.  `interleaved=True` pairs (x[2i], x[2i+1])
as RoFormer prints it; `interleaved=False` pairs (x[i], x[i + d/2]), the split-halves layout of the
public Llama / Qwen model code, and is the default reading.
"""
import numpy as np


def angles(n, d, base=10000.0, pos0=0):
    """[n, d/2] fp64: (pos0 + m) * base^(-2 i / d)."""
    assert d % 2 == 0
    m = np.arange(pos0, pos0 + n, dtype=np.float64)[:, None]
    theta = np.float64(base) ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)
    return m * theta[None, :]


def rope(X, base=10000.0, pos0=0, interleaved=False, inverse=False):
    """X: [..., n, d] (any leading dims); row m of every leading slice sits at position pos0 + m.
    inverse=True rotates by the negative angle (the transpose of the rotation: what the backward
    pass applies to the gradients of the rotated Q and K)."""
    X = np.asarray(X, dtype=np.float64)
    n, d = X.shape[-2], X.shape[-1]
    ang = angles(n, d, base, pos0)
    c, s = np.cos(ang), np.sin(ang)
    if inverse:
        s = -s
    out = np.empty_like(X)
    if interleaved:
        a, b = X[..., 0::2], X[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = a * s + b * c
    else:
        h = d // 2
        a, b = X[..., :h], X[..., h:]
        out[..., :h] = a * c - b * s
        out[..., h:] = a * s + b * c
    return out
