"""GPU parity of sa_bwd (ungated and gated) against the fp64 oracle's analytic gradient."""
import numpy as np
import pytest
import torch

from tests import gpu_util as U

pytestmark = pytest.mark.gpu

CIRC, LIN, ONE = 0, 1, 2


def grad_close(got, ref, dtype, what):
    # max-abs bar scaled by the reference's own magnitude (gradients are not O(1) like Y)
    U.assert_close(got, ref, dtype, what, scale_abs=max(1.0, float(np.abs(ref).max())))


def run_bwd(B, Hq, Hkv, n, d, w, window, causal, dtype, perm_B=1, perm_H=1, seed=0, identity=False,
            k_growth=0.0):
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    wl, x = U.make_case(B, Hq, Hkv, n, d, w, dtype, perm_B, perm_H, seed, grads=True, identity=identity)
    if k_growth:  # keys grow with their original position: later (masked) keys outscore the visible ones
        from paper_2604_00754_amd import synth
        ramp = (1.0 + k_growth * np.arange(n, dtype=np.float32) / n)[None, None, :, None]
        x["K"] = (x["K"] * ramp).astype(np.float32)
        if dtype == "bf16":
            x["K"] = synth.round_to_bf16(x["K"])
    print(f"case bwd B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} w{w} win{window} causal{causal} {dtype} "
          f"perm[{perm_B},{perm_H}] identity={identity}", flush=True)
    oc = U.orc_desc(wl, window, causal)
    dQr, dKr, dVr = orc.sa_bwd(oc, x["Q"], x["K"], x["V"], x["perm"], x["dY"])
    Q, K, V, dY = (U.to_dev(x[k], dtype) for k in ("Q", "K", "V", "dY"))
    perm = None if identity else torch.from_numpy(x["perm"]).to(U.DEV)
    desc = U.sa_desc(wl, window, causal)
    Y = torch.empty_like(Q)
    L = torch.empty((B, Hq, n), device=U.DEV, dtype=torch.float32)
    sa.sa_fwd(desc, Q, K, V, perm, Y, L)
    dQ, dK, dV = torch.full_like(Q, float("nan")), torch.full_like(K, float("nan")), torch.full_like(V, float("nan"))
    # the workspace enters as NaN bit patterns: whatever a kernel reads from it (the row sums the dQ kernel leaves for
    # the dK/dV kernel) must have been written by the same call
    ws = torch.full((sa.sa_workspace_bytes(desc, sa.SA_OP_BWD),), 255, device=U.DEV, dtype=torch.uint8)
    sa.sa_bwd(desc, None, Q, K, V, perm, None, None, Y, None, L, None, dY, dQ, dK, dV, None, None, ws)
    torch.cuda.synchronize()
    grad_close(U.to_np64(dQ), dQr, dtype, "dQ")
    grad_close(U.to_np64(dK), dKr, dtype, "dK")
    grad_close(U.to_np64(dV), dVr, dtype, "dV")


def run_gated_bwd(B, Hq, Hkv, n, d, w, dtype, perm_B=1, perm_H=1, per_dim=0, gate_dtype="f32", seed=0):
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    wl, x = U.make_case(B, Hq, Hkv, n, d, w, dtype, perm_B, perm_H, seed, gates=True, grads=True)
    print(f"case gated bwd B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} w{w} {dtype} perm[{perm_B},{perm_H}] "
          f"per_dim={per_dim} gate={gate_dtype}", flush=True)
    ga, gl = x["gate_sa"], x["gate_swa"]
    if per_dim:
        rng = np.random.default_rng(seed)
        ga = rng.standard_normal((B, Hq, n, d)).astype(np.float32)
        gl = rng.standard_normal((B, Hq, n, d)).astype(np.float32)
    if gate_dtype == "bf16":
        ga, gl = synth.round_to_bf16(ga), synth.round_to_bf16(gl)
    osa, oswa = U.orc_desc(wl, CIRC, 1), U.orc_desc(wl, ONE, 1)
    ref = orc.gated_sa_swa_bwd(osa, oswa, per_dim, x["Q"], x["K"], x["V"], x["perm"], ga, gl, x["dY"])
    Q, K, V, dY = (U.to_dev(x[k], dtype) for k in ("Q", "K", "V", "dY"))
    perm = torch.from_numpy(x["perm"]).to(U.DEV)
    gdt = 1 if gate_dtype == "f32" else 0
    tga, tgl = U.to_dev(ga, gate_dtype), U.to_dev(gl, gate_dtype)
    dsa, dswa = U.sa_desc(wl, CIRC, 1, per_dim, gdt), U.sa_desc(wl, ONE, 1, per_dim, gdt)
    Y, Ysa, Yswa = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)
    Lsa = torch.empty((B, Hq, n), device=U.DEV, dtype=torch.float32)
    Lswa = torch.empty_like(Lsa)
    wsf = torch.empty(max(sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_FWD), 16), device=U.DEV, dtype=torch.uint8)
    sa.gated_sa_swa_fwd(dsa, dswa, Q, K, V, perm, tga, tgl, Y, Ysa, Yswa, Lsa, Lswa, wsf)
    dQ, dK, dV = torch.full_like(Q, float("nan")), torch.full_like(K, float("nan")), torch.full_like(V, float("nan"))
    dga, dgl = torch.full_like(tga, float("nan")), torch.full_like(tgl, float("nan"))
    ws = torch.full((sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_BWD),), 255, device=U.DEV, dtype=torch.uint8)
    sa.sa_bwd(dsa, dswa, Q, K, V, perm, tga, tgl, Ysa, Yswa, Lsa, Lswa, dY, dQ, dK, dV, dga, dgl, ws)
    torch.cuda.synchronize()
    for got, r, what in ((dQ, ref[0], "dQ"), (dK, ref[1], "dK"), (dV, ref[2], "dV")):
        grad_close(U.to_np64(got), r, dtype, what)
    gtol = "bf16" if (dtype == "bf16" or gate_dtype == "bf16") else "f32"
    grad_close(U.to_np64(dga), ref[3], gtol, "dgate_sa")
    grad_close(U.to_np64(dgl), ref[4], gtol, "dgate_swa")


@pytest.mark.parametrize("window,causal", [(CIRC, 1), (CIRC, 0), (LIN, 1), (ONE, 1)])
def test_bwd_f32(window, causal):
    run_bwd(1, 4, 2, 300, 64, 37, window, causal, "f32", perm_H=4, seed=1)


def test_bwd_f32_d128_and_full_ring():
    run_bwd(1, 2, 2, 150, 128, 64, CIRC, 1, "f32", seed=2)
    run_bwd(1, 2, 1, 90, 64, 200, CIRC, 1, "f32", seed=3)
    run_bwd(1, 2, 2, 130, 64, 16, ONE, 1, "f32", seed=4, identity=True)


@pytest.mark.parametrize("per_dim", [0, 1])
def test_gated_bwd_f32(per_dim):
    run_gated_bwd(1, 4, 2, 200, 64, 32, "f32", perm_H=4, per_dim=per_dim, seed=5)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("window,causal", [(CIRC, 1), (CIRC, 0), (LIN, 1), (ONE, 1)])
def test_bwd_bf16(d, window, causal):
    run_bwd(2, 4, 2, 700, d, 128, window, causal, "bf16", seed=10 + d)


@pytest.mark.parametrize("n,w", [(77, 16), (129, 300), (640, 641), (300, 1), (31, 64), (513, 2)])
def test_bwd_bf16_ragged_and_degenerate(n, w):
    run_bwd(1, 2, 2, n, 64, w, CIRC, 1, "bf16", seed=20)
    run_bwd(1, 2, 1, n, 128, w, CIRC, 0, "bf16", seed=21)


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (4, 2), (6, 2), (3, 1), (16, 2)])
def test_bwd_bf16_query_heads_of_a_group_share_a_workgroup(Hq, Hkv):
    """One permutation for all heads (or none): the dQ kernel processes the query heads of a KV group 4, 2 or 1
    at a time over the same slots, by group size (4, 2, 3, 3 and 8 here).  Ragged n, several window kinds."""
    run_bwd(1, Hq, Hkv, 555, 128, 128, CIRC, 1, "bf16", seed=80 + Hq)
    run_bwd(2, Hq, Hkv, 300, 64, 70, LIN, 0, "bf16", perm_B=2, seed=81 + Hq)
    run_bwd(1, Hq, Hkv, 421, 64, 64, ONE, 1, "bf16", identity=True, seed=82 + Hq)
    run_bwd(1, Hq, Hkv, 31, 64, 8, CIRC, 1, "bf16", seed=83 + Hq)


@pytest.mark.parametrize("n", [1, 33, 64, 65, 127, 128, 129, 191, 257])
def test_bwd_bf16_slot_counts_around_tile_edges(n):
    """Sequence lengths around multiples of the 32-slot blocks and of the 64- / 128-slot streamed tiles."""
    for d in (64, 128):
        run_bwd(1, 4, 1, n, d, 40, CIRC, 1, "bf16", seed=95 + d)
        run_bwd(1, 2, 2, n, d, 2 * n + 3, CIRC, 1, "bf16", perm_H=2, seed=96 + d)
        run_bwd(1, 1, 1, n, d, 64, ONE, 1, "bf16", identity=True, seed=97 + d)


def test_bwd_bf16_per_head_perm_with_grouped_heads():
    run_bwd(2, 8, 2, 600, 64, 128, CIRC, 1, "bf16", perm_B=2, perm_H=8, seed=30)
    run_bwd(1, 4, 4, 600, 64, 128, CIRC, 1, "bf16", perm_H=4, seed=31)


@pytest.mark.parametrize("per_dim,gate_dtype", [(0, "f32"), (1, "f32"), (0, "bf16")])
def test_gated_bwd_bf16(per_dim, gate_dtype):
    run_gated_bwd(2, 4, 2, 700, 64, 128, "bf16", per_dim=per_dim, gate_dtype=gate_dtype, seed=40)


def test_gated_bwd_bf16_d128():
    run_gated_bwd(1, 4, 1, 500, 128, 96, "bf16", seed=41)


def test_bwd_bf16_later_keys_dominate():
    """Scores of later (causally masked) keys far above the visible ones: in the 16-bit causal mode
    exp(score - LSE) of such a pair is many orders of magnitude above one before the packed mask clears
    it, and must leave no trace in dQ, dK, dV.  (The growth is kept where the visible scores stay benign:
    a steeper ramp makes the softmax of late rows one-hot and the bf16 gradient itself ill-conditioned,
    rel-L2 5.0e-3 at a ramp of 10.)"""
    run_bwd(1, 2, 2, 1500, 64, 256, CIRC, 1, "bf16", seed=70, k_growth=4.0)
    run_bwd(1, 2, 1, 900, 128, 128, CIRC, 1, "bf16", perm_H=2, seed=71, k_growth=3.0)


@pytest.mark.parametrize("n", [65535, 65536])
def test_bwd_bf16_index_width_boundary(n):
    """The largest n of the 16-bit causal mode and the first n of the 32-bit mode, both backward kernels."""
    run_bwd(1, 1, 1, n, 64, 32, CIRC, 1, "bf16", seed=72)
    run_bwd(1, 2, 1, n, 128, 32, ONE, 1, "bf16", seed=73, identity=True)
