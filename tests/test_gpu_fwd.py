"""GPU parity of the forward entry points (sa_fwd, swa_fwd) against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from tests import gpu_util as U

pytestmark = pytest.mark.gpu

CIRC, LIN, ONE = 0, 1, 2


def run_fwd(B, Hq, Hkv, n, d, w, window, causal, dtype, perm_B=1, perm_H=1, seed=0, identity=False,
            use_swa_entry=False, k_growth=0.0):
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    wl, x = U.make_case(B, Hq, Hkv, n, d, w, dtype, perm_B, perm_H, seed, identity=identity)
    if k_growth:  # keys grow with their original position: later (masked) keys outscore the visible ones
        from paper_2604_00754_amd import synth
        ramp = (1.0 + k_growth * np.arange(n, dtype=np.float32) / n)[None, None, :, None]
        x["K"] = (x["K"] * ramp).astype(np.float32)
        if dtype == "bf16":
            x["K"] = synth.round_to_bf16(x["K"])
    print(f"case fwd B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} w{w} win{window} causal{causal} {dtype} "
          f"perm[{perm_B},{perm_H}] identity={identity}", flush=True)
    Yr, Lr = orc.sa_fwd(U.orc_desc(wl, window, causal), x["Q"], x["K"], x["V"], x["perm"])
    Q, K, V = (U.to_dev(x[k], dtype) for k in "QKV")
    perm = None if identity else torch.from_numpy(x["perm"]).to(U.DEV)
    Y = torch.full_like(Q, float("nan"))
    L = torch.full((B, Hq, n), float("nan"), device=U.DEV, dtype=torch.float32)
    desc = U.sa_desc(wl, window, causal)
    if use_swa_entry:
        sa.swa_fwd(desc, Q, K, V, Y, L)
    else:
        sa.sa_fwd(desc, Q, K, V, perm, Y, L)
    torch.cuda.synchronize()
    U.assert_close(U.to_np64(Y), Yr, dtype, "Y")
    la = np.abs(U.to_np64(L) - Lr).max()
    assert la <= (4e-3 if dtype == "bf16" else 1e-5), f"LSE max-abs {la:.3e}"
    if causal:
        # the token at original position 0 sees itself only (Sec. 3.3: causal on original positions), whatever the
        # window and wherever it sits in the permuted order: its output is its own V row, bit for bit -- one masked
        # key that leaked with any weight would change it
        g = Hq // Hkv
        for hq in range(Hq):
            assert torch.equal(Y[:, hq, 0, :], V[:, hq // g, 0, :]), f"head {hq}: row of original position 0"


def test_tiny_f32_config():
    """First benchmark configuration: B=1, H=2, n=1024, d=64, w=64, fp32, one permutation per head."""
    run_fwd(1, 2, 2, 1024, 64, 64, CIRC, 1, "f32", perm_H=2)


@pytest.mark.parametrize("window", [CIRC, LIN, ONE])
@pytest.mark.parametrize("causal", [0, 1])
def test_f32_window_kinds(window, causal):
    run_fwd(2, 4, 2, 333, 64, 37, window, causal, "f32", perm_B=2, perm_H=4, seed=1)


def test_f32_d128_and_wide_windows():
    run_fwd(1, 2, 1, 200, 128, 64, CIRC, 1, "f32", seed=2)
    run_fwd(1, 2, 1, 150, 128, 151, CIRC, 1, "f32", seed=3)     # window covers the ring
    run_fwd(1, 1, 1, 150, 64, 400, ONE, 1, "f32", seed=4, identity=True, use_swa_entry=True)
    run_fwd(1, 1, 1, 70, 64, 1, CIRC, 1, "f32", seed=5)         # w = 1: every token sees itself only


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("window,causal", [(CIRC, 1), (CIRC, 0), (LIN, 1), (ONE, 1)])
def test_bf16_basic(d, window, causal):
    run_fwd(2, 4, 2, 1000, d, 128, window, causal, "bf16", perm_H=4, seed=10 + d)


@pytest.mark.parametrize("n,w", [(77, 16), (128, 9), (129, 300), (640, 641), (1024, 1023), (300, 1), (31, 64), (513, 2)])
def test_bf16_ragged_and_degenerate(n, w):
    run_fwd(1, 2, 2, n, 64, w, CIRC, 1, "bf16", seed=20)
    run_fwd(1, 2, 1, n, 128, w, CIRC, 0, "bf16", perm_H=2, seed=21)
    run_fwd(1, 2, 1, n, 128, w, LIN, 1, "bf16", seed=22)


def test_bf16_swa_entry_and_identity():
    run_fwd(2, 4, 4, 900, 64, 128, ONE, 1, "bf16", identity=True, use_swa_entry=True, seed=30)
    run_fwd(1, 4, 1, 900, 128, 100, ONE, 1, "bf16", identity=True, use_swa_entry=True, seed=31)
    run_fwd(1, 2, 2, 900, 64, 128, CIRC, 1, "bf16", identity=True, seed=32)
    run_fwd(1, 2, 2, 500, 64, 2000, ONE, 1, "bf16", identity=True, use_swa_entry=True, seed=33)  # full causal


def test_bf16_gqa_shared_and_per_batch_perm():
    run_fwd(2, 8, 2, 1100, 128, 256, CIRC, 1, "bf16", perm_B=2, perm_H=1, seed=40)
    run_fwd(2, 8, 2, 600, 64, 256, CIRC, 1, "bf16", perm_B=2, perm_H=8, seed=41)


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (4, 2), (16, 2), (6, 2), (3, 1), (12, 2)])
def test_bf16_query_heads_of_a_group_share_a_workgroup(Hq, Hkv):
    """One permutation for all heads (or none): the query heads of a KV group are processed 4, 2 or 1 at
    a time over the same slots, by group size (4, 2, 8, 3, 3 and 6 here).  Ragged n (not a multiple of 32),
    each window kind, d = 64 and 128; per-head permutations keep one head per workgroup."""
    run_fwd(1, Hq, Hkv, 555, 128, 128, CIRC, 1, "bf16", seed=60 + Hq)
    run_fwd(2, Hq, Hkv, 300, 64, 70, LIN, 0, "bf16", perm_B=2, seed=61 + Hq)
    run_fwd(1, Hq, Hkv, 421, 64, 64, ONE, 1, "bf16", identity=True, use_swa_entry=True, seed=62 + Hq)
    run_fwd(1, Hq, Hkv, 333, 128, 500, CIRC, 1, "bf16", perm_H=Hq, seed=63 + Hq)   # window covers the ring
    run_fwd(1, Hq, Hkv, 31, 64, 8, CIRC, 1, "bf16", seed=64 + Hq)                  # less than one wave of slots


@pytest.mark.parametrize("n", [1, 2, 32, 33, 63, 64, 65, 96, 97, 159, 160, 161, 255, 257])
def test_bf16_slot_counts_around_tile_edges(n):
    """Sequence lengths around multiples of the 32-slot blocks and of the 32- / 64-key tiles (d = 128 / 64),
    with windows below, at and above n, each window kind, with and without shared workgroups."""
    for d in (64, 128):
        run_fwd(1, 4, 1, n, d, 40, CIRC, 1, "bf16", seed=90 + d)                     # four heads per workgroup
        run_fwd(1, 2, 2, n, d, 2 * n + 3, CIRC, 1, "bf16", perm_H=2, seed=91 + d)   # window covers the ring
        run_fwd(1, 2, 1, n, d, 33, LIN, 0, "bf16", seed=92 + d)                     # two heads per workgroup
        run_fwd(1, 1, 1, n, d, 64, ONE, 1, "bf16", identity=True, use_swa_entry=True, seed=93 + d)


def test_bf16_later_keys_dominate():
    """Scores of later (causally masked) keys far above the visible ones: the packed 16-bit mask clears
    their probabilities after the exponential, so they must neither move the softmax reference nor leak
    an overflow into the row sums."""
    run_fwd(1, 2, 2, 1500, 64, 256, CIRC, 1, "bf16", seed=50, k_growth=40.0)
    run_fwd(1, 2, 1, 900, 128, 128, CIRC, 1, "bf16", perm_H=2, seed=51, k_growth=25.0)


@pytest.mark.parametrize("shift", [150.0, -150.0, 0.0, 30.0, -30.0])
@pytest.mark.parametrize("d,causal", [(128, 1), (64, 1), (64, 0)])
def test_bf16_scores_far_from_zero(shift, d, causal):
    """The kernel first runs a band with the softmax reference fixed at zero and goes through it again with the
    running maximum when a row sum leaves the range of that form.  Scores around +150 (every exponential
    overflows), around -150 (every exponential underflows) and rows of both kinds side by side in one workgroup
    (shift 0 here: the sign alternates with the original position) must all come out as the oracle's
    max-subtracted softmax does; so must scores around +-30, which the zero-reference form still holds (row sums
    near 2^43 and 2^-43)."""
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    B, Hq, Hkv, n, w = 1, 4, 2, 700, 128
    wl, x = U.make_case(B, Hq, Hkv, n, d, w, "bf16", 1, 1, seed=90 + d)
    rng = np.random.default_rng(5)
    u = rng.standard_normal(d).astype(np.float32)
    u /= np.linalg.norm(u)
    target = 150.0 if shift == 0.0 else abs(shift)
    amp = np.sqrt(target * np.sqrt(d))         # (amp u) . (amp u) / sqrt(d) = target
    sign = np.where(np.arange(n) % 2 == 0, 1.0, -1.0) if shift == 0.0 else np.full(n, np.sign(shift))
    x["Q"] = synth.round_to_bf16((x["Q"] + (sign[:, None] * amp * u)[None, None]).astype(np.float32))
    x["K"] = synth.round_to_bf16((x["K"] + (amp * u)[None, None, None]).astype(np.float32))
    print(f"case fwd far-from-zero shift{shift} d{d} causal{causal}", flush=True)
    Yr, Lr = orc.sa_fwd(U.orc_desc(wl, CIRC, causal), x["Q"], x["K"], x["V"], x["perm"])
    if target == 150.0:
        assert np.abs(Lr).min() > 60.0         # the rows really are out of the zero-reference form's range
    else:
        assert 12.0 < np.abs(Lr).min() and np.abs(Lr).max() < 52.0   # and these inside it (ln 2^80 = 55.5)
    Q, K, V = (U.to_dev(x[k], "bf16") for k in "QKV")
    perm = torch.from_numpy(x["perm"]).to(U.DEV)
    Y = torch.full_like(Q, float("nan"))
    L = torch.full((B, Hq, n), float("nan"), device=U.DEV, dtype=torch.float32)
    sa.sa_fwd(U.sa_desc(wl, CIRC, causal), Q, K, V, perm, Y, L)
    torch.cuda.synchronize()
    U.assert_close(U.to_np64(Y), Yr, "bf16", "Y")
    # LSE is of order 150 here: its fp32 representation alone has steps of 1.5e-5, the bf16 bar applies on top
    assert np.abs(U.to_np64(L) - Lr).max() <= 4e-3 + 1e-4


def test_bf16_long_sequence_uses_32bit_indices():
    """n > 65535: original positions no longer fit the 16-bit mask path."""
    run_fwd(1, 1, 1, 66000, 64, 64, CIRC, 1, "bf16", seed=52)


@pytest.mark.parametrize("n", [65535, 65536])
def test_bf16_index_width_boundary(n):
    """The largest n of the 16-bit causal mode (original positions up to 65534, biased to int16) and the
    first n of the 32-bit mode."""
    run_fwd(1, 1, 1, n, 64, 32, CIRC, 1, "bf16", seed=53)
    run_fwd(1, 1, 1, n, 128, 32, ONE, 1, "bf16", seed=54, identity=True, use_swa_entry=True)


def test_pretraining_shape_sample():
    """Second benchmark configuration's shape (B=8,H=12,n=2048,d=64,w=128), SA branch only."""
    run_fwd(8, 12, 12, 2048, 64, 128, CIRC, 1, "bf16", perm_H=12, seed=50)


def test_check_perm_accepts_bijections_and_rejects_others():
    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth
    B, H, n = 2, 3, 1000
    desc = sa.make_desc(B, H, H, n, 64, 32, perm_B=B, perm_H=H)
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_CHECK_PERM), device=U.DEV, dtype=torch.uint8)
    good = torch.from_numpy(synth.permutations(B, H, n)).to(U.DEV)
    sa.sa_check_perm(desc, good, ws)
    sa.sa_check_perm(desc, good, ws)  # the workspace is cleared by the call itself
    for bad_value in (good[0, 0, 5].item(), -1, n):
        bad = good.clone()
        bad[1, 2, 7] = bad_value if bad_value != good[1, 2, 7].item() else good[1, 2, 8].item()
        with pytest.raises(sa.SaError) as e:
            sa.sa_check_perm(desc, bad, ws)
        assert e.value.status == sa.SA_ERR_BAD_PERM


@pytest.mark.parametrize("d,Hq,Hkv,perm_H", [(128, 4, 2, 1), (64, 6, 2, 6), (64, 2, 2, 1)])
def test_permuted_copy_moves_every_row_once(d, Hq, Hkv, perm_H):
    """sa_permuted_copy (gather + scatter without attention): bit-exact against the same sums formed
    with torch in fp32 and rounded once; ragged n so that the last lane groups are partly idle."""
    from paper_2604_00754_amd import binding as sa
    B, n = 2, 1237
    wl, x = U.make_case(B, Hq, Hkv, n, d, 64, "bf16", 1, perm_H, seed=60 + d)
    Q, K, V = (U.to_dev(x[k], "bf16") for k in "QKV")
    perm = torch.from_numpy(x["perm"]).to(U.DEV)
    Y = torch.full_like(Q, float("nan"))
    sa.sa_permuted_copy(U.sa_desc(wl, CIRC, 1), Q, K, V, perm, Y)
    torch.cuda.synchronize()
    g = Hq // Hkv
    ref = Q.float().clone()
    ref[:, ::g] += K.float() + V.float()
    assert torch.equal(Y, ref.to(torch.bfloat16))
    Y2 = torch.full_like(Q, float("nan"))
    sa.sa_permuted_copy(U.sa_desc(wl, CIRC, 1), Q, K, V, None, Y2)  # identity: same result, contiguous order
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y)
