"""GPU parity of sa_rope_table / sa_rope (RoPE on original positions, App. B, App. C / Sec. 4.2; RoFormer Sec. 3.2.2)
against the fp64 numpy oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def gpu_table(n, d, base, pos0):
    from paper_2604_00754_amd import binding as sa
    t = torch.full((n, d // 2, 2), float("nan"), device=U.DEV, dtype=torch.float32)
    sa.sa_rope_table(n, d, base, pos0, t)
    torch.cuda.synchronize()
    return t


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("base,pos0", [(1e4, 0), (1e6, 0), (1e4, 131072 - 333), (1e6, 2_000_000)])
def test_table_matches_fp64_angles(d, base, pos0):
    from oracle import rope as R
    n = 333
    print(f"case rope_table n{n} d{d} base{base} pos0 {pos0}", flush=True)
    t = gpu_table(n, d, base, pos0).cpu().numpy().astype(np.float64)
    ang = R.angles(n, d, base, pos0)
    # fp32 rounding of a value in [-1, 1] (6e-8) plus the fp64 angle error (|angle| * 2^-52 * few)
    assert np.abs(t[..., 0] - np.cos(ang)).max() <= 2e-7
    assert np.abs(t[..., 1] - np.sin(ang)).max() <= 2e-7


def run_apply(B, Hq, Hkv, n, d, dtype, interleaved, base=1e4, pos0=0, seed=0, in_place=False):
    from oracle import rope as R
    from paper_2604_00754_amd import binding as sa
    print(f"case rope B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} {dtype} interleaved={interleaved} base={base} pos0={pos0} "
          f"in_place={in_place}", flush=True)
    wl, x = U.make_case(B, Hq, Hkv, n, d, 4, dtype, seed=seed, identity=True)
    Q, K = U.to_dev(x["Q"], dtype), U.to_dev(x["K"], dtype)
    q64, k64 = U.to_np64(Q), U.to_np64(K)     # what the kernel reads (bf16-rounded for bf16)
    table = gpu_table(n, d, base, pos0)
    desc = sa.make_desc(B, Hq, Hkv, n, d, 4, dtype=sa.SA_BF16 if dtype == "bf16" else sa.SA_F32)
    Qo = Q if in_place else torch.full_like(Q, float("nan"))
    Ko = K if in_place else torch.full_like(K, float("nan"))
    sa.sa_rope(desc, Q, K, table, Qo, Ko, interleaved=interleaved)
    torch.cuda.synchronize()
    kw = dict(base=base, pos0=pos0, interleaved=bool(interleaved))
    rq, rk = R.rope(q64, **kw), R.rope(k64, **kw)
    U.assert_close(U.to_np64(Qo), rq, dtype, "rope(Q)")
    U.assert_close(U.to_np64(Ko), rk, dtype, "rope(K)")
    # inverse: the backward of the rotation, applied to a gradient
    g = U.to_dev(np.random.default_rng(seed + 9).standard_normal(x["Q"].shape).astype(np.float32), dtype)
    go = torch.full_like(g, float("nan"))
    sa.sa_rope(desc, g, None, table, go, None, interleaved=interleaved, inverse=1)
    torch.cuda.synchronize()
    U.assert_close(U.to_np64(go), R.rope(U.to_np64(g), inverse=True, **kw), dtype, "rope^T(dQ)")
    return Qo, Ko


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("interleaved", [0, 1])
def test_rope_apply(dtype, d, interleaved):
    run_apply(2, 4, 2, 301, d, dtype, interleaved, seed=d + interleaved)   # ragged last block, GQA


def test_rope_in_place_many_heads_and_late_positions():
    run_apply(1, 9, 3, 130, 64, "bf16", 0, in_place=True, seed=3)          # head count not a multiple of 4
    run_apply(1, 2, 1, 200, 128, "bf16", 0, base=1e6, pos0=131072 - 200, seed=4)
    run_apply(1, 2, 1, 200, 128, "f32", 1, base=1e6, pos0=131072 - 200, seed=5)
    run_apply(1, 1, 1, 1, 64, "f32", 0, seed=6)                            # a single row at position 0: identity


def test_rope_then_attention_matches_the_oracle_composition():
    """fp32 end to end: rotate Q and K on original positions, then SA forward and backward, then the inverse
    rotation of dQ and dK; against rope -> attention -> rope^T of the oracle."""
    from oracle import binding as orc
    from oracle import rope as R
    from paper_2604_00754_amd import binding as sa
    B, Hq, Hkv, n, d, w = 1, 4, 2, 260, 64, 32
    print(f"case rope+sa B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} w{w} f32", flush=True)
    wl, x = U.make_case(B, Hq, Hkv, n, d, w, "f32", seed=21, grads=True)
    c = U.orc_desc(wl, 0, 1)
    rq, rk = R.rope(x["Q"]), R.rope(x["K"])
    Yr, _ = orc.sa_fwd(c, rq, rk, x["V"], x["perm"])
    dq, dk, dv = orc.sa_bwd(c, rq, rk, x["V"], x["perm"], x["dY"])
    dq, dk = R.rope(dq, inverse=True), R.rope(dk, inverse=True)
    Q, K, V, dY = (U.to_dev(x[k], "f32") for k in ("Q", "K", "V", "dY"))
    perm = torch.from_numpy(x["perm"]).to(U.DEV)
    desc = U.sa_desc(wl, 0, 1)
    table = gpu_table(n, d, 1e4, 0)
    Qr, Kr = torch.empty_like(Q), torch.empty_like(K)
    sa.sa_rope(desc, Q, K, table, Qr, Kr)
    Y = torch.full_like(Q, float("nan"))
    L = torch.empty((B, Hq, n), device=U.DEV)
    sa.sa_fwd(desc, Qr, Kr, V, perm, Y, L)
    dQ, dK, dV = torch.full_like(Q, float("nan")), torch.full_like(K, float("nan")), torch.full_like(V, float("nan"))
    ws = torch.full((sa.sa_workspace_bytes(desc, sa.SA_OP_BWD),), 255, device=U.DEV, dtype=torch.uint8)
    sa.sa_bwd(desc, None, Qr, Kr, V, perm, None, None, Y, None, L, None, dY, dQ, dK, dV, None, None, ws)
    sa.sa_rope(desc, dQ, dK, table, dQ, dK, inverse=1)
    torch.cuda.synchronize()
    U.assert_close(U.to_np64(Y), Yr, "f32", "Y")
    for name, got, ref in (("dQ", dQ, dq), ("dK", dK, dk), ("dV", dV, dv)):
        U.assert_close(U.to_np64(got), ref, "f32", name, scale_abs=max(1.0, float(np.abs(ref).max())))


def test_rope_rejects_bad_arguments():
    from paper_2604_00754_amd import binding as sa
    t = torch.zeros((8, 32, 2), device=U.DEV)
    x = torch.zeros((1, 1, 8, 64), device=U.DEV, dtype=torch.bfloat16)
    desc = sa.make_desc(1, 1, 1, 8, 64, 4)
    for args, status in (((8, 96, 1e4, 0, t), sa.SA_ERR_UNSUPPORTED), ((8, 64, 1.0, 0, t), sa.SA_ERR_SHAPE),
                         ((0, 64, 1e4, 0, t), sa.SA_ERR_SHAPE), ((8, 64, 1e4, -1, t), sa.SA_ERR_SHAPE),
                         ((8, 64, 1e4, 0, None), sa.SA_ERR_NULL)):
        with pytest.raises(sa.SaError) as e:
            sa.sa_rope_table(*args)
        assert e.value.status == status
    with pytest.raises(sa.SaError) as e:
        sa.sa_rope(desc, x, None, t, None, None)      # Q without an output
    assert e.value.status == sa.SA_ERR_NULL
    with pytest.raises(sa.SaError) as e:
        sa.sa_rope(desc, x, None, t, x, None, interleaved=2)
    assert e.value.status == sa.SA_ERR_SHAPE


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("interleaved", [0, 1])
def test_forward_with_fused_query_rotation(d, interleaved):
    """sa_fwd_rope (Q rotated on original positions while it is staged, K rotated in memory by sa_rope)
    against rope -> attention of the oracle in fp64, and against the unfused GPU path."""
    from oracle import binding as orc
    from oracle import rope as R
    from paper_2604_00754_amd import binding as sa
    B, Hq, Hkv, n, w = 2, 4, 2, 700, 128
    for identity, window in ((False, 0), (True, 2)):
        print(f"case fwd_rope B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} w{w} interleaved={interleaved} identity={identity}",
              flush=True)
        wl, x = U.make_case(B, Hq, Hkv, n, d, w, "bf16", 1, 1 if identity else Hq, seed=80 + d + interleaved,
                            identity=identity)
        Q, K, V = (U.to_dev(x[k], "bf16") for k in "QKV")
        kw = dict(base=1e4, pos0=0, interleaved=bool(interleaved))
        # in the bf16 configuration the rotated rows are bf16 values (that is where both GPU paths round):
        # the oracle rotates in fp64 and rounds to bf16 with the input generator's rounding routine
        from paper_2604_00754_amd import synth
        rq = synth.round_to_bf16(R.rope(U.to_np64(Q), **kw).astype(np.float32))
        rk = synth.round_to_bf16(R.rope(U.to_np64(K), **kw).astype(np.float32))
        Yr, Lr = orc.sa_fwd(U.orc_desc(wl, window, 1), rq, rk, U.to_np64(V), x["perm"])
        perm = None if identity else torch.from_numpy(x["perm"]).to(U.DEV)
        desc = U.sa_desc(wl, window, 1)
        table = gpu_table(n, d, 1e4, 0)
        Kr, Qr = torch.empty_like(K), torch.empty_like(Q)
        sa.sa_rope(desc, None, K, table, None, Kr, interleaved=interleaved)
        Y = torch.full_like(Q, float("nan"))
        L = torch.full((B, Hq, n), float("nan"), device=U.DEV)
        sa.sa_fwd_rope(desc, Q, Kr, V, perm, table, Y, L, interleaved=interleaved)
        sa.sa_rope(desc, Q, None, table, Qr, None, interleaved=interleaved)
        Y2 = torch.full_like(Q, float("nan"))
        sa.sa_fwd(desc, Qr, Kr, V, perm, Y2, None)
        torch.cuda.synchronize()
        U.assert_close(U.to_np64(Y), Yr, "bf16", "Y (fused rotation)")
        assert np.abs(U.to_np64(L) - Lr).max() <= 4e-3
        # the two GPU paths round the rotated Q to bf16 at the same point; they may differ by how the
        # compiler contracts a*c - b*s, i.e. by single bf16 steps of single Q elements
        U.assert_close(U.to_np64(Y), U.to_np64(Y2), "bf16", "fused vs unfused")


def test_fwd_rope_rejects_unsupported():
    from paper_2604_00754_amd import binding as sa
    t = torch.zeros((8, 32, 2), device=U.DEV)
    x = torch.zeros((1, 1, 8, 64), device=U.DEV, dtype=torch.float32)
    with pytest.raises(sa.SaError) as e:
        sa.sa_fwd_rope(sa.make_desc(1, 1, 1, 8, 64, 4, dtype=sa.SA_F32), x, x, x, None, t, torch.empty_like(x))
    assert e.value.status == sa.SA_ERR_UNSUPPORTED
    xb = x.to(torch.bfloat16)
    with pytest.raises(sa.SaError) as e:
        sa.sa_fwd_rope(sa.make_desc(1, 1, 1, 8, 64, 4), xb, xb, xb, None, None, torch.empty_like(xb))
    assert e.value.status == sa.SA_ERR_NULL


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("interleaved", [0, 1])
@pytest.mark.parametrize("dk_unrotated", [0, 1])
def test_backward_with_fused_rotations(d, interleaved, dk_unrotated):
    """sa_bwd_rope (Q rotated while the dQ kernel stages it, dQ -- and on request dK -- turned back in the
    epilogues) against rope -> analytic gradient -> rope^T of the oracle in fp64."""
    from oracle import binding as orc
    from oracle import rope as R
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    B, Hq, Hkv, n, w = 2, 4, 2, 700, 128
    # shared permutation; one permutation per query head (one dK/dV pass per head of a group, summed in place);
    # identity order with the one-sided window (the SWA branch)
    for identity, window, perm_H in ((False, 0, 1), (False, 0, Hq), (True, 2, 1)):
        print(f"case bwd_rope B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} w{w} interleaved={interleaved} dk_unrotated={dk_unrotated} "
              f"identity={identity} perm_H={perm_H}", flush=True)
        wl, x = U.make_case(B, Hq, Hkv, n, d, w, "bf16", 1, perm_H, seed=300 + d + interleaved, grads=True,
                            identity=identity)
        Q, K, V, dY = (U.to_dev(x[k], "bf16") for k in ("Q", "K", "V", "dY"))
        kw = dict(base=1e4, pos0=0, interleaved=bool(interleaved))
        # as in the forward, the rotated rows are bf16 values on both sides
        rq = synth.round_to_bf16(R.rope(U.to_np64(Q), **kw).astype(np.float32))
        rk = synth.round_to_bf16(R.rope(U.to_np64(K), **kw).astype(np.float32))
        oc = U.orc_desc(wl, window, 1)
        dq, dk, dv = orc.sa_bwd(oc, rq, rk, U.to_np64(V), x["perm"], U.to_np64(dY))
        dq = R.rope(dq, inverse=True, **kw)
        if dk_unrotated:
            dk = R.rope(dk, inverse=True, **kw)
        perm = None if identity else torch.from_numpy(x["perm"]).to(U.DEV)
        desc = U.sa_desc(wl, window, 1)
        table = gpu_table(n, d, 1e4, 0)
        Kr = torch.empty_like(K)
        sa.sa_rope(desc, None, K, table, None, Kr, interleaved=interleaved)
        Y = torch.empty_like(Q)
        L = torch.empty((B, Hq, n), device=U.DEV)
        sa.sa_fwd_rope(desc, Q, Kr, V, perm, table, Y, L, interleaved=interleaved)
        dQ, dK, dV = (torch.full_like(t, float("nan")) for t in (Q, K, V))
        ws = torch.full((sa.sa_workspace_bytes(desc, sa.SA_OP_BWD_ROPE),), 255, device=U.DEV, dtype=torch.uint8)
        Q0 = Q.clone()
        sa.sa_bwd_rope(desc, Q, Kr, V, perm, table, Y, L, dY, dQ, dK, dV, ws, interleaved=interleaved,
                       dk_unrotated=dk_unrotated)
        torch.cuda.synchronize()
        assert torch.equal(Q, Q0)     # the rotated rows go to the workspace, not over the input
        for name, got, ref in (("dQ", dQ, dq), ("dK", dK, dk), ("dV", dV, dv)):
            U.assert_close(U.to_np64(got), ref, "bf16", name, scale_abs=max(1.0, float(np.abs(ref).max())))


def test_bwd_rope_rejects_unsupported():
    from paper_2604_00754_amd import binding as sa
    t = torch.zeros((8, 32, 2), device=U.DEV)
    xb = torch.zeros((1, 1, 8, 64), device=U.DEV, dtype=torch.bfloat16)
    L = torch.zeros((1, 1, 8), device=U.DEV)
    desc = sa.make_desc(1, 1, 1, 8, 64, 4)
    ws = torch.full((sa.sa_workspace_bytes(desc, sa.SA_OP_BWD_ROPE),), 255, device=U.DEV, dtype=torch.uint8)
    out = [torch.empty_like(xb) for _ in range(3)]
    with pytest.raises(sa.SaError) as e:   # no table
        sa.sa_bwd_rope(desc, xb, xb, xb, None, None, xb, L, xb, *out, ws)
    assert e.value.status == sa.SA_ERR_NULL
    with pytest.raises(sa.SaError) as e:   # workspace of the plain backward: too small for the rotated rows
        sa.sa_bwd_rope(desc, xb, xb, xb, None, t, xb, L, xb, *out, ws[:sa.sa_workspace_bytes(desc, sa.SA_OP_BWD)])
    assert e.value.status == sa.SA_ERR_WORKSPACE
    with pytest.raises(sa.SaError) as e:
        sa.sa_bwd_rope(desc, xb, xb, xb, None, t, xb, L, xb, *out, ws, dk_unrotated=2)
    assert e.value.status == sa.SA_ERR_SHAPE
    xf = xb.float()
    with pytest.raises(sa.SaError) as e:
        sa.sa_bwd_rope(sa.make_desc(1, 1, 1, 8, 64, 4, dtype=sa.SA_F32), xf, xf, xf, None, t, xf, L, xf,
                       *[torch.empty_like(xf) for _ in range(3)], ws)
    assert e.value.status == sa.SA_ERR_UNSUPPORTED
