"""GPU parity of sa_dual_path_fwd / sa_dual_path_bwd (the whole layer of Alg. 2: stochastic branch, sliding-window
branch, Eq. 6 gates over the model dimension, Eq. 5 sum) against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from tests import gpu_util as U

pytestmark = pytest.mark.gpu

CIRC, ONE = 0, 2


def run_layer(B, Hq, Hkv, n, d, w, perm_H=1, seed=0, backward=True, train=True):
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    dm = Hq * d
    print(f"case dual_path B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} w{w} perm_H{perm_H} bwd={backward} train={train}", flush=True)
    wl, x = U.make_case(B, Hq, Hkv, n, d, w, "bf16", 1, perm_H, seed, grads=True)
    rng = np.random.default_rng(synth.BASE_SEED + 500 + seed)
    Wsa, Wswa = (synth.round_to_bf16((rng.standard_normal((dm, dm)) / np.sqrt(dm) * 2).astype(np.float32))
                 for _ in range(2))
    osa, oswa = U.orc_desc(wl, CIRC, 1), U.orc_desc(wl, ONE, 1)
    ref = orc.dual_path_fwd(osa, oswa, x["Q"], x["K"], x["V"], x["perm"], Wsa, Wswa)
    dev = lambda a: U.to_dev(a, "bf16")
    Q, K, V, tWa, tWb = dev(x["Q"]), dev(x["K"]), dev(x["V"]), dev(Wsa), dev(Wswa)
    perm = torch.from_numpy(x["perm"]).to(U.DEV)
    nan = lambda t: torch.full_like(t, float("nan"))
    Y, Ya, Yb = nan(Q), nan(Q), nan(Q)
    Ga, Gb = (nan(Q), nan(Q)) if train else (None, None)
    La, Lb = ((torch.full((B, Hq, n), float("nan"), device=U.DEV) for _ in range(2))) if train else (None, None)
    dsa, dswa = U.sa_desc(wl, CIRC, 1), U.sa_desc(wl, ONE, 1)
    sa.sa_dual_path_fwd(dsa, dswa, Q, K, V, perm, tWa, tWb, Y, Ya, Yb, Ga, Gb, La, Lb)
    torch.cuda.synchronize()
    U.assert_close(U.to_np64(Y), ref["Y"], "bf16", "Y")
    U.assert_close(U.to_np64(Ya), ref["Ysa"], "bf16", "Y_sa")
    U.assert_close(U.to_np64(Yb), ref["Yswa"], "bf16", "Y_swa")
    if train:
        sig = lambda z: 1 / (1 + np.exp(-z))
        U.assert_close(U.to_np64(Ga), sig(ref["Lsa"]), "bf16", "G_sa")
        U.assert_close(U.to_np64(Gb), sig(ref["Lswa"]), "bf16", "G_swa")
        assert np.abs(U.to_np64(La) - ref["LSEsa"]).max() <= 4e-3
        assert np.abs(U.to_np64(Lb) - ref["LSEswa"]).max() <= 4e-3
    if not backward:
        return
    rb = orc.dual_path_bwd(osa, oswa, x["Q"], x["K"], x["V"], x["perm"], Wsa, Wswa, x["dY"])
    dY = dev(x["dY"])
    dQ, dK, dV, dWa, dWb = nan(Q), nan(K), nan(V), nan(tWa), nan(tWb)
    ws = torch.full((sa.sa_workspace_bytes(dsa, sa.SA_OP_DUAL_PATH_BWD),), 255, device=U.DEV, dtype=torch.uint8)
    sa.sa_dual_path_bwd(dsa, dswa, Q, K, V, perm, tWa, tWb, Ya, Yb, Ga, Gb, La, Lb, dY, dQ, dK, dV, dWa, dWb, ws)
    torch.cuda.synchronize()
    for name, got in (("dQ", dQ), ("dK", dK), ("dV", dV), ("dWsa", dWa), ("dWswa", dWb)):
        r = rb[name]
        U.assert_close(U.to_np64(got), r, "bf16", name, scale_abs=max(1.0, float(np.abs(r).max())))
    with pytest.raises(sa.SaError) as e:
        sa.sa_dual_path_bwd(dsa, dswa, Q, K, V, perm, tWa, tWb, Ya, Yb, Ga, Gb, La, Lb, dY, dQ, dK, dV, dWa, dWb,
                            ws[:-256])
    assert e.value.status == sa.SA_ERR_WORKSPACE


@pytest.mark.parametrize("d,Hq,Hkv", [(64, 4, 2), (128, 2, 1)])
def test_dual_path_layer_forward_and_backward(d, Hq, Hkv):
    run_layer(2, Hq, Hkv, 600, d, 128, perm_H=Hq, seed=d)      # ragged tiles, per-head permutations


def test_dual_path_layer_inference_mode():
    run_layer(1, 4, 4, 520, 64, 64, seed=3, backward=False, train=False)


def test_dual_path_layer_pretraining_shape():
    """Heads, head size and window of the pre-training setup (App. B / App. C: 16 heads of 64, w = 256), short n."""
    run_layer(1, 16, 16, 1024, 64, 256, seed=4)


def test_dual_path_rejects_unsupported():
    from paper_2604_00754_amd import binding as sa
    t = torch.zeros((1, 1, 8, 64), device=U.DEV, dtype=torch.bfloat16)
    w = torch.zeros((64, 64), device=U.DEV, dtype=torch.bfloat16)
    p = torch.arange(8, device=U.DEV, dtype=torch.int32).reshape(1, 1, 8)
    dsa = sa.make_desc(1, 1, 1, 8, 64, 4, CIRC, 1)
    dswa = sa.make_desc(1, 1, 1, 8, 64, 4, ONE, 1)
    with pytest.raises(sa.SaError) as e:   # model dimension 64 is not a multiple of 128
        sa.sa_dual_path_fwd(dsa, dswa, t, t, t, p, w, w, torch.empty_like(t), torch.empty_like(t),
                            torch.empty_like(t))
    assert e.value.status == sa.SA_ERR_UNSUPPORTED
