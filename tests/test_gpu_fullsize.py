"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the GPU result
is compared with the fp64 oracle on a seeded sample of output rows (rows are independent, so the
oracle computes exactly those rows one by one)."""
import numpy as np
import pytest
import torch

from tests import gpu_util as U

pytestmark = pytest.mark.gpu

CIRC, LIN, ONE = 0, 1, 2


def gpu_normal(shape, seed, dtype=torch.bfloat16):
    g = torch.Generator(device=U.DEV)
    g.manual_seed(seed)
    return torch.randn(shape, device=U.DEV, dtype=torch.float32, generator=g).to(dtype)


def host64(t):
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


def pick(t, rows):
    ri = torch.from_numpy(rows.astype(np.int64)).to(t.device)
    return host64(t[ri[:, 0], ri[:, 1], ri[:, 2]])


def fwd_fullsize(name, rows_per_head):
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    wl = synth.WORKLOADS[name]
    print(f"case fullsize fwd {name}", flush=True)
    Q = gpu_normal((wl.B, wl.Hq, wl.n, wl.d), 1)
    K = gpu_normal((wl.B, wl.Hkv, wl.n, wl.d), 2)
    V = gpu_normal((wl.B, wl.Hkv, wl.n, wl.d), 3)
    perm_np = synth.permutations(wl.perm_B, wl.perm_H, wl.n)
    perm = torch.from_numpy(perm_np).to(U.DEV)
    Q64, K64, V64 = host64(Q), host64(K), host64(V)
    rows = synth.sample_rows(wl.B, wl.Hq, wl.n, rows_per_head, seed=11)
    # make sure the sample meets the ragged ends of the slot range (first/last tiles, wrap-around)
    edge = np.array([(0, h, int(perm_np[0, 0, p])) for h in range(wl.Hq) for p in (0, 1, wl.n - 1)], np.int32)
    rows = np.concatenate([rows, edge])
    Y = torch.full_like(Q, float("nan"))
    L = torch.full((wl.B, wl.Hq, wl.n), float("nan"), device=U.DEV, dtype=torch.float32)
    for window, use_perm in ((CIRC, True), (ONE, False)):
        desc = U.sa_desc(wl, window, 1)
        if use_perm:
            sa.sa_fwd(desc, Q, K, V, perm, Y, L)
        else:
            sa.swa_fwd(desc, Q, K, V, Y, L)
        torch.cuda.synchronize()
        assert torch.isfinite(Y.float()).all().item() and torch.isfinite(L).all().item()
        Yr, Lr = orc.sa_fwd_rows(U.orc_desc(wl, window, 1), Q64, K64, V64, perm_np if use_perm else None, rows)
        ma, rl = U.assert_close(pick(Y, rows), Yr, "bf16", f"{name} Y rows (window {window})")
        ri = torch.from_numpy(rows.astype(np.int64)).to(U.DEV)
        la = np.abs(L[ri[:, 0], ri[:, 1], ri[:, 2]].cpu().numpy().astype(np.float64) - Lr).max()
        assert la <= 4e-3, la
        print(f"  window {window}: {rows.shape[0]} rows max-abs {ma:.2e} rel-L2 {rl:.2e} lse {la:.1e}", flush=True)


def test_qwen3_8b_prefill_32k_sampled_rows():
    fwd_fullsize("qwen3_8b_prefill_32k", 24)


def test_qwen3_30b_prefill_128k_sampled_rows():
    fwd_fullsize("qwen3_30b_prefill_128k", 6)


def test_pretrain_fwdbwd_8k_gated_sampled_rows():
    """Fourth benchmark configuration: B=4, H=16, n=8192, d=64, w=256, gated SA+SWA forward and
    backward, one permutation per layer shared by the heads."""
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    wl = synth.WORKLOADS["pretrain_fwdbwd_8k"]
    print("case fullsize gated fwd+bwd pretrain_fwdbwd_8k", flush=True)
    B, H, n, d = wl.B, wl.Hq, wl.n, wl.d
    Q, K, V, dY = (gpu_normal((B, H, n, d), s) for s in (1, 2, 3, 4))
    ga = gpu_normal((B, H, n), 5, torch.float32)
    gl = gpu_normal((B, H, n), 6, torch.float32)
    perm_np = synth.permutations(1, 1, n)
    perm = torch.from_numpy(perm_np).to(U.DEV)
    dsa, dswa = U.sa_desc(wl, CIRC, 1), U.sa_desc(wl, ONE, 1)
    Y, Ysa, Yswa = (torch.full_like(Q, float("nan")) for _ in range(3))
    Lsa = torch.empty((B, H, n), device=U.DEV, dtype=torch.float32)
    Lswa = torch.empty_like(Lsa)
    wsf = torch.empty(sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_FWD), device=U.DEV, dtype=torch.uint8)
    sa.gated_sa_swa_fwd(dsa, dswa, Q, K, V, perm, ga, gl, Y, Ysa, Yswa, Lsa, Lswa, wsf)
    dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(3))
    dga, dgl = torch.full_like(ga, float("nan")), torch.full_like(gl, float("nan"))
    ws = torch.empty(sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_BWD), device=U.DEV, dtype=torch.uint8)
    sa.sa_bwd(dsa, dswa, Q, K, V, perm, ga, gl, Ysa, Yswa, Lsa, Lswa, dY, dQ, dK, dV, dga, dgl, ws)
    torch.cuda.synchronize()
    for t in (Y, Ysa, Yswa, dQ, dK, dV, dga, dgl):
        assert torch.isfinite(t.float()).all().item()

    Q64, K64, V64, dY64, ga64, gl64 = (host64(t) for t in (Q, K, V, dY, ga, gl))
    osa, oswa = U.orc_desc(wl, CIRC, 1), U.orc_desc(wl, ONE, 1)
    rows = synth.sample_rows(B, H, n, 6, seed=12)
    m = rows.shape[0]
    rdesc = orc.desc(1, 1, 1, m, d, 1)                      # the sampled rows seen as one small tensor
    Ysa_r, _ = orc.sa_fwd_rows(osa, Q64, K64, V64, perm_np, rows)
    Yswa_r, _ = orc.sa_fwd_rows(oswa, Q64, K64, V64, None, rows)
    ga_r = ga64[rows[:, 0], rows[:, 1], rows[:, 2]].reshape(1, 1, m)
    gl_r = gl64[rows[:, 0], rows[:, 1], rows[:, 2]].reshape(1, 1, m)
    Y_r = orc.gate_combine(rdesc, 0, Ysa_r.reshape(1, 1, m, d), Yswa_r.reshape(1, 1, m, d), ga_r, gl_r)
    U.assert_close(pick(Y, rows), Y_r.reshape(m, d), "bf16", "Y rows")
    U.assert_close(pick(Ysa, rows), Ysa_r, "bf16", "Y_sa rows")
    U.assert_close(pick(Yswa, rows), Yswa_r, "bf16", "Y_swa rows")

    # backward: Eq. 5's chain rule on the full dY (element-wise, cheap), then row-sampled gradients
    fdesc = orc.desc(B, H, H, n, d, wl.w)
    dYsa, dYswa = orc.gate_bwd(fdesc, 0, dY64, ga64, gl64)
    dQ_r = orc.sa_bwd_dq_rows(osa, Q64, K64, V64, perm_np, dYsa, rows) + \
        orc.sa_bwd_dq_rows(oswa, Q64, K64, V64, None, dYswa, rows)
    scale = lambda r: max(1.0, float(np.abs(r).max()))
    U.assert_close(pick(dQ, rows), dQ_r, "bf16", "dQ rows", scale_abs=scale(dQ_r))
    krows = synth.sample_rows(B, H, n, 2, seed=13)
    dKa, dVa = orc.sa_bwd_dkv_rows(osa, Q64, K64, V64, perm_np, dYsa, krows)
    dKl, dVl = orc.sa_bwd_dkv_rows(oswa, Q64, K64, V64, None, dYswa, krows)
    U.assert_close(pick(dK, krows), dKa + dKl, "bf16", "dK rows", scale_abs=scale(dKa + dKl))
    U.assert_close(pick(dV, krows), dVa + dVl, "bf16", "dV rows", scale_abs=scale(dVa + dVl))
    dY_r = dY64[rows[:, 0], rows[:, 1], rows[:, 2]].reshape(1, 1, m, d)
    _, _, dga_r, dgl_r = orc.gate_bwd(rdesc, 0, dY_r, ga_r, gl_r, Ysa_r.reshape(1, 1, m, d), Yswa_r.reshape(1, 1, m, d))
    ri = torch.from_numpy(rows.astype(np.int64)).to(U.DEV)
    for got, ref, what in ((dga, dga_r, "dgate_sa"), (dgl, dgl_r, "dgate_swa")):
        g = got[ri[:, 0], ri[:, 1], ri[:, 2]].cpu().numpy().astype(np.float64)
        U.assert_close(g, ref.reshape(m), "bf16", what + " rows", scale_abs=scale(ref))
