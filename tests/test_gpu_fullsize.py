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


EDGE_SLOTS = (0, 1, 31, 32, 63, 64, 127, 128, -129, -128, -33, -32, -1)


def edge_rows(perm_np, B, H, n, heads=None):
    """(b, h, original index) of the tokens that sit at the first and last permuted slots and on both sides of the
    32-, 64- and 128-slot tile edges: the rows whose bands wrap around and meet the ragged ends of the tiling."""
    heads = range(H) if heads is None else heads
    out = [(b, h, int(perm_np[0, 0, p % n])) for b in range(B) for h in heads for p in EDGE_SLOTS]
    return np.array(out, np.int32)


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
    rows = np.concatenate([rows, edge_rows(perm_np, wl.B, wl.Hq, wl.n)])
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
    fwd_fullsize("qwen3_30b_prefill_128k", 64)


def test_qwen3_8b_prefill_32k_backward_sampled_rows():
    """sa_bwd at the headline shape (d = 128, grouped heads 4:1, n = 32768, w = 512), the call bench.py times as
    `sa_bwd_headline_shape`: dQ on sampled query rows, dK and dV on sampled key rows of every KV head, against the
    row-wise fp64 gradients of the oracle."""
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    wl = synth.WORKLOADS["qwen3_8b_prefill_32k"]
    print("case fullsize bwd qwen3_8b_prefill_32k", flush=True)
    B, Hq, Hkv, n, d = wl.B, wl.Hq, wl.Hkv, wl.n, wl.d
    Q = gpu_normal((B, Hq, n, d), 1)
    K = gpu_normal((B, Hkv, n, d), 2)
    V = gpu_normal((B, Hkv, n, d), 3)
    dY = gpu_normal((B, Hq, n, d), 4)
    perm_np = synth.permutations(1, 1, n)
    perm = torch.from_numpy(perm_np).to(U.DEV)
    desc = U.sa_desc(wl, CIRC, 1)
    Y = torch.full_like(Q, float("nan"))
    L = torch.full((B, Hq, n), float("nan"), device=U.DEV, dtype=torch.float32)
    sa.sa_fwd(desc, Q, K, V, perm, Y, L)
    dQ = torch.full_like(Q, float("nan"))
    dK, dV = torch.full_like(K, float("nan")), torch.full_like(K, float("nan"))
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_BWD), device=U.DEV, dtype=torch.uint8)
    sa.sa_bwd(desc, None, Q, K, V, perm, None, None, Y, None, L, None, dY, dQ, dK, dV, None, None, ws)
    torch.cuda.synchronize()
    for t in (dQ, dK, dV):
        assert torch.isfinite(t.float()).all().item()
    Q64, K64, V64, dY64 = (host64(t) for t in (Q, K, V, dY))
    od = U.orc_desc(wl, CIRC, 1)
    scale = lambda r: max(1.0, float(np.abs(r).max()))
    rows = np.concatenate([synth.sample_rows(B, Hq, n, 16, seed=21), edge_rows(perm_np, B, Hq, n)])
    dQ_r = orc.sa_bwd_dq_rows(od, Q64, K64, V64, perm_np, dY64, rows)
    ma, rl = U.assert_close(pick(dQ, rows), dQ_r, "bf16", "dQ rows", scale_abs=scale(dQ_r))
    print(f"  dQ: {rows.shape[0]} rows max-abs {ma:.2e} rel-L2 {rl:.2e}", flush=True)
    krows = np.concatenate([synth.sample_rows(B, Hkv, n, 8, seed=22), edge_rows(perm_np, B, Hkv, n)])
    dK_r, dV_r = orc.sa_bwd_dkv_rows(od, Q64, K64, V64, perm_np, dY64, krows)
    ma, rl = U.assert_close(pick(dK, krows), dK_r, "bf16", "dK rows", scale_abs=scale(dK_r))
    print(f"  dK: {krows.shape[0]} rows max-abs {ma:.2e} rel-L2 {rl:.2e}", flush=True)
    ma, rl = U.assert_close(pick(dV, krows), dV_r, "bf16", "dV rows", scale_abs=scale(dV_r))
    print(f"  dV: {krows.shape[0]} rows max-abs {ma:.2e} rel-L2 {rl:.2e}", flush=True)


def test_qwen3_8b_prefill_32k_fused_query_rotation_sampled_rows():
    """rope(K) in memory + sa_fwd_rope (Q rotated while it is staged) at the headline shape with the Qwen3 base
    10^6, the pair of calls bench.py times as `rope_k_plus_fwd_rope`: sampled rows against rope -> attention of
    the oracle, whose rotated rows are rounded to bf16 where both GPU paths round."""
    from oracle import binding as orc
    from oracle import rope as R
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    wl = synth.WORKLOADS["qwen3_8b_prefill_32k"]
    print("case fullsize fwd_rope qwen3_8b_prefill_32k", flush=True)
    B, Hq, Hkv, n, d = wl.B, wl.Hq, wl.Hkv, wl.n, wl.d
    Q = gpu_normal((B, Hq, n, d), 1)
    K = gpu_normal((B, Hkv, n, d), 2)
    V = gpu_normal((B, Hkv, n, d), 3)
    perm_np = synth.permutations(1, 1, n)
    perm = torch.from_numpy(perm_np).to(U.DEV)
    desc = U.sa_desc(wl, CIRC, 1)
    table = torch.empty((n, d // 2, 2), device=U.DEV, dtype=torch.float32)
    sa.sa_rope_table(n, d, 1e6, 0, table)
    Kr = torch.empty_like(K)
    sa.sa_rope(desc, None, K, table, None, Kr)
    Y = torch.full_like(Q, float("nan"))
    L = torch.full((B, Hq, n), float("nan"), device=U.DEV, dtype=torch.float32)
    sa.sa_fwd_rope(desc, Q, Kr, V, perm, table, Y, L)
    torch.cuda.synchronize()
    assert torch.isfinite(Y.float()).all().item() and torch.isfinite(L).all().item()
    rq = synth.round_to_bf16(R.rope(host64(Q), base=1e6).astype(np.float32)).astype(np.float64)
    rk = synth.round_to_bf16(R.rope(host64(K), base=1e6).astype(np.float32)).astype(np.float64)
    rows = np.concatenate([synth.sample_rows(B, Hq, n, 16, seed=23), edge_rows(perm_np, B, Hq, n)])
    Yr, Lr = orc.sa_fwd_rows(U.orc_desc(wl, CIRC, 1), rq, rk, host64(V), perm_np, rows)
    ma, rl = U.assert_close(pick(Y, rows), Yr, "bf16", "Y rows (fused rotation)")
    ri = torch.from_numpy(rows.astype(np.int64)).to(U.DEV)
    la = np.abs(L[ri[:, 0], ri[:, 1], ri[:, 2]].cpu().numpy().astype(np.float64) - Lr).max()
    assert la <= 4e-3, la
    print(f"  {rows.shape[0]} rows max-abs {ma:.2e} rel-L2 {rl:.2e} lse {la:.1e}", flush=True)


def test_qwen3_8b_prefill_32k_backward_with_fused_rotations_sampled_rows():
    """sa_bwd_rope at the headline shape with the Qwen3 base 10^6 and dK turned back, the call bench.py times as
    `sa_bwd_rope`: dQ on sampled query rows, dK and dV on sampled key rows, against rope -> row-wise fp64 gradients
    -> rope^T of the oracle (the inverse rotation of a row needs that row only)."""
    from oracle import binding as orc
    from oracle import rope as R
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    wl = synth.WORKLOADS["qwen3_8b_prefill_32k"]
    print("case fullsize bwd_rope qwen3_8b_prefill_32k", flush=True)
    B, Hq, Hkv, n, d = wl.B, wl.Hq, wl.Hkv, wl.n, wl.d
    Q = gpu_normal((B, Hq, n, d), 1)
    K = gpu_normal((B, Hkv, n, d), 2)
    V = gpu_normal((B, Hkv, n, d), 3)
    dY = gpu_normal((B, Hq, n, d), 4)
    perm_np = synth.permutations(1, 1, n)
    perm = torch.from_numpy(perm_np).to(U.DEV)
    desc = U.sa_desc(wl, CIRC, 1)
    table = torch.empty((n, d // 2, 2), device=U.DEV, dtype=torch.float32)
    sa.sa_rope_table(n, d, 1e6, 0, table)
    Kr = torch.empty_like(K)
    sa.sa_rope(desc, None, K, table, None, Kr)
    Y = torch.full_like(Q, float("nan"))
    L = torch.full((B, Hq, n), float("nan"), device=U.DEV, dtype=torch.float32)
    sa.sa_fwd_rope(desc, Q, Kr, V, perm, table, Y, L)
    dQ = torch.full_like(Q, float("nan"))
    dK, dV = torch.full_like(K, float("nan")), torch.full_like(K, float("nan"))
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_BWD_ROPE), device=U.DEV, dtype=torch.uint8)
    sa.sa_bwd_rope(desc, Q, Kr, V, perm, table, Y, L, dY, dQ, dK, dV, ws, dk_unrotated=1)
    torch.cuda.synchronize()
    for t in (dQ, dK, dV):
        assert torch.isfinite(t.float()).all().item()
    rq = synth.round_to_bf16(R.rope(host64(Q), base=1e6).astype(np.float32)).astype(np.float64)
    rk = synth.round_to_bf16(R.rope(host64(K), base=1e6).astype(np.float32)).astype(np.float64)
    V64, dY64 = host64(V), host64(dY)
    od = U.orc_desc(wl, CIRC, 1)
    ang = R.angles(n, d, 1e6, 0)

    def turn_back(rows_grad, positions):  # rope^T of single rows (split-halves pairing), each at its own position
        c, sn = np.cos(ang[positions]), np.sin(ang[positions])
        a, b = rows_grad[:, :d // 2], rows_grad[:, d // 2:]
        return np.concatenate([a * c + b * sn, b * c - a * sn], axis=1)

    scale = lambda r: max(1.0, float(np.abs(r).max()))
    rows = np.concatenate([synth.sample_rows(B, Hq, n, 16, seed=31), edge_rows(perm_np, B, Hq, n)])
    dQ_r = turn_back(orc.sa_bwd_dq_rows(od, rq, rk, V64, perm_np, dY64, rows), rows[:, 2])
    ma, rl = U.assert_close(pick(dQ, rows), dQ_r, "bf16", "dQ rows (fused rotations)", scale_abs=scale(dQ_r))
    print(f"  dQ: {rows.shape[0]} rows max-abs {ma:.2e} rel-L2 {rl:.2e}", flush=True)
    krows = np.concatenate([synth.sample_rows(B, Hkv, n, 8, seed=32), edge_rows(perm_np, B, Hkv, n)])
    dK_r, dV_r = orc.sa_bwd_dkv_rows(od, rq, rk, V64, perm_np, dY64, krows)
    dK_r = turn_back(dK_r, krows[:, 2])
    ma, rl = U.assert_close(pick(dK, krows), dK_r, "bf16", "dK rows (fused rotations)", scale_abs=scale(dK_r))
    print(f"  dK: {krows.shape[0]} rows max-abs {ma:.2e} rel-L2 {rl:.2e}", flush=True)
    ma, rl = U.assert_close(pick(dV, krows), dV_r, "bf16", "dV rows (fused rotations)", scale_abs=scale(dV_r))
    print(f"  dV: {krows.shape[0]} rows max-abs {ma:.2e} rel-L2 {rl:.2e}", flush=True)


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
    rows = np.concatenate([synth.sample_rows(B, H, n, 6, seed=12), edge_rows(perm_np, B, H, n, heads=(0, 5, H - 1)),
                           np.array([(b, h, i) for b in (0, B - 1) for h in (0, H - 1) for i in (0, 1, 255, 256, n - 1)], np.int32)])
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
    krows = np.concatenate([synth.sample_rows(B, H, n, 2, seed=13), edge_rows(perm_np, B, H, n, heads=(0, H - 1)),
                            np.array([(0, 3, i) for i in (0, 127, 128, n - 256, n - 1)], np.int32)])
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


def test_pretrain_fwdbwd_8k_single_path_whole_tensors():
    """The shape the backward's roofline block is quoted on (B=4, H=16, n=8192, d=64, w=256, one permutation shared by
    the heads), single-path sa_fwd + sa_bwd in the launch configuration bench.py times: every element of Y, LSE, dQ,
    dK and dV against the oracle (about ten seconds of CPU work)."""
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    wl = synth.WORKLOADS["pretrain_fwdbwd_8k"]
    print("case fullsize whole tensors sa_fwd + sa_bwd pretrain_fwdbwd_8k", flush=True)
    B, H, n, d = wl.B, wl.Hq, wl.n, wl.d
    Q, K, V, dY = (gpu_normal((B, H, n, d), s) for s in (11, 12, 13, 14))
    perm_np = synth.permutations(1, 1, n)
    perm = torch.from_numpy(perm_np).to(U.DEV)
    desc = U.sa_desc(wl, CIRC, 1)
    Y = torch.full_like(Q, float("nan"))
    L = torch.full((B, H, n), float("nan"), device=U.DEV, dtype=torch.float32)
    sa.sa_fwd(desc, Q, K, V, perm, Y, L)
    dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(3))
    ws = torch.full((sa.sa_workspace_bytes(desc, sa.SA_OP_BWD),), 255, device=U.DEV, dtype=torch.uint8)
    sa.sa_bwd(desc, None, Q, K, V, perm, None, None, Y, None, L, None, dY, dQ, dK, dV, None, None, ws)
    torch.cuda.synchronize()
    Q64, K64, V64, dY64 = (host64(t) for t in (Q, K, V, dY))
    oc = U.orc_desc(wl, CIRC, 1)
    Yr, Lr = orc.sa_fwd(oc, Q64, K64, V64, perm_np)
    U.assert_close(U.to_np64(Y), Yr, "bf16", "Y")
    assert np.abs(L.cpu().numpy().astype(np.float64) - Lr).max() <= 4e-3, "LSE"
    dQr, dKr, dVr = orc.sa_bwd(oc, Q64, K64, V64, perm_np, dY64)
    for got, ref, what in ((dQ, dQr, "dQ"), (dK, dKr, "dK"), (dV, dVr, "dV")):
        U.assert_close(U.to_np64(got), ref, "bf16", what, scale_abs=max(1.0, float(np.abs(ref).max())))


def test_pretrain_fwdbwd_8k_gated_whole_tensors():
    """Fourth benchmark configuration whole: gated SA + SWA forward and backward at B=4, H=16, n=8192, d=64, w=256 in
    the launch configuration bench.py times, every element of Y, Y_sa, Y_swa, dQ, dK, dV and both gate gradients
    against the oracle (the sampled-row test above names rows; this one leaves none out)."""
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    wl = synth.WORKLOADS["pretrain_fwdbwd_8k"]
    print("case fullsize whole tensors gated fwd + bwd pretrain_fwdbwd_8k", flush=True)
    B, H, n, d = wl.B, wl.Hq, wl.n, wl.d
    Q, K, V, dY = (gpu_normal((B, H, n, d), s) for s in (21, 22, 23, 24))
    ga = gpu_normal((B, H, n), 25, torch.float32)
    gl = gpu_normal((B, H, n), 26, torch.float32)
    perm_np = synth.permutations(1, 1, n)
    perm = torch.from_numpy(perm_np).to(U.DEV)
    dsa, dswa = U.sa_desc(wl, CIRC, 1), U.sa_desc(wl, ONE, 1)
    Y, Ysa, Yswa = (torch.full_like(Q, float("nan")) for _ in range(3))
    Lsa = torch.empty((B, H, n), device=U.DEV, dtype=torch.float32)
    Lswa = torch.empty_like(Lsa)
    wsf = torch.full((sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_FWD),), 255, device=U.DEV, dtype=torch.uint8)
    sa.gated_sa_swa_fwd(dsa, dswa, Q, K, V, perm, ga, gl, Y, Ysa, Yswa, Lsa, Lswa, wsf)
    dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(3))
    dga, dgl = torch.full_like(ga, float("nan")), torch.full_like(gl, float("nan"))
    ws = torch.full((sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_BWD),), 255, device=U.DEV, dtype=torch.uint8)
    sa.sa_bwd(dsa, dswa, Q, K, V, perm, ga, gl, Ysa, Yswa, Lsa, Lswa, dY, dQ, dK, dV, dga, dgl, ws)
    torch.cuda.synchronize()
    Q64, K64, V64, dY64, ga64, gl64 = (host64(t) for t in (Q, K, V, dY, ga, gl))
    osa, oswa = U.orc_desc(wl, CIRC, 1), U.orc_desc(wl, ONE, 1)
    f = orc.gated_sa_swa_fwd(osa, oswa, 0, Q64, K64, V64, perm_np, ga64, gl64)
    U.assert_close(U.to_np64(Y), f["Y"], "bf16", "Y")
    U.assert_close(U.to_np64(Ysa), f["Ysa"], "bf16", "Y_sa")
    U.assert_close(U.to_np64(Yswa), f["Yswa"], "bf16", "Y_swa")
    del f
    ref = orc.gated_sa_swa_bwd(osa, oswa, 0, Q64, K64, V64, perm_np, ga64, gl64, dY64)
    for got, r, what in ((dQ, ref[0], "dQ"), (dK, ref[1], "dK"), (dV, ref[2], "dV"), (dga, ref[3], "dgate_sa"),
                         (dgl, ref[4], "dgate_swa")):
        U.assert_close(U.to_np64(got), r, "bf16", what, scale_abs=max(1.0, float(np.abs(r).max())))


def test_qwen3_8b_prefill_32k_forward_backward_whole_tensors():
    """The headline shape whole (B=1, 32 / 8 heads, n=32768, d=128, w=512): every element of Y, LSE, dQ, dK and dV of
    sa_fwd + sa_bwd against the oracle (about twenty seconds of CPU work on the GPU machine's cores)."""
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    wl = synth.WORKLOADS["qwen3_8b_prefill_32k"]
    print("case fullsize whole tensors sa_fwd + sa_bwd qwen3_8b_prefill_32k", flush=True)
    B, Hq, Hkv, n, d = wl.B, wl.Hq, wl.Hkv, wl.n, wl.d
    Q, dY = gpu_normal((B, Hq, n, d), 31), gpu_normal((B, Hq, n, d), 34)
    K, V = gpu_normal((B, Hkv, n, d), 32), gpu_normal((B, Hkv, n, d), 33)
    perm_np = synth.permutations(1, 1, n)
    perm = torch.from_numpy(perm_np).to(U.DEV)
    desc = U.sa_desc(wl, CIRC, 1)
    Y = torch.full_like(Q, float("nan"))
    L = torch.full((B, Hq, n), float("nan"), device=U.DEV, dtype=torch.float32)
    sa.sa_fwd(desc, Q, K, V, perm, Y, L)
    dQ = torch.full_like(Q, float("nan"))
    dK, dV = torch.full_like(K, float("nan")), torch.full_like(K, float("nan"))
    ws = torch.full((sa.sa_workspace_bytes(desc, sa.SA_OP_BWD),), 255, device=U.DEV, dtype=torch.uint8)
    sa.sa_bwd(desc, None, Q, K, V, perm, None, None, Y, None, L, None, dY, dQ, dK, dV, None, None, ws)
    torch.cuda.synchronize()
    Q64, K64, V64, dY64 = (host64(t) for t in (Q, K, V, dY))
    od = U.orc_desc(wl, CIRC, 1)
    Yr, Lr = orc.sa_fwd(od, Q64, K64, V64, perm_np)
    U.assert_close(U.to_np64(Y), Yr, "bf16", "Y")
    assert np.abs(L.cpu().numpy().astype(np.float64) - Lr).max() <= 4e-3, "LSE"
    del Yr, Lr
    dQr, dKr, dVr = orc.sa_bwd(od, Q64, K64, V64, perm_np, dY64)
    for got, ref, what in ((dQ, dQr, "dQ"), (dK, dKr, "dK"), (dV, dVr, "dV")):
        U.assert_close(U.to_np64(got), ref, "bf16", what, scale_abs=max(1.0, float(np.abs(ref).max())))
