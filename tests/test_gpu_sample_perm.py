"""GPU parity of sa_sample_perm (on-device permutation sampling, Sec. 3.3) against the numpy oracle:
bit-exact, since both sides sort the same SplitMix64 keys."""
import numpy as np
import pytest
import torch

from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def sample(B, H, perm_B, perm_H, n, seed, layer, workspace=False):
    """workspace=False: the O(n^2) rank count; True: the bucketed O(n) path with its workspace."""
    from paper_2604_00754_amd import binding as sa
    desc = sa.make_desc(B, H, H, n, 64, 8, perm_B=perm_B, perm_H=perm_H)
    perm = torch.full((perm_B, perm_H, n), -1, device=U.DEV, dtype=torch.int32)
    ws = None
    if workspace:  # filled with ones: the call must clear what it counts in
        ws = torch.full((sa.sa_workspace_bytes(desc, sa.SA_OP_SAMPLE_PERM),), 0xFF, device=U.DEV, dtype=torch.uint8)
    sa.sa_sample_perm(desc, seed, layer, perm, ws)
    torch.cuda.synchronize()
    return desc, perm


@pytest.mark.parametrize("n", [1, 5, 256, 1000, 1024, 4097, 16384, 20011, 32768])
def test_sample_perm_matches_oracle_bit_for_bit(n):
    from oracle import perm_sampler as ps
    print(f"case sample_perm n{n}", flush=True)
    for perm_B, perm_H, seed, layer in ((1, 1, 0, 0), (2, 3, 20260400754, 5)):
        ref = ps.sample_perm(seed, layer, perm_B, perm_H, n)
        for workspace in (False, True):
            _, perm = sample(2, 3, perm_B, perm_H, n, seed, layer, workspace)
            assert np.array_equal(perm.cpu().numpy(), ref), f"workspace={workspace}"


def test_sample_perm_long_sequence_and_full_64_bit_seed():
    from oracle import perm_sampler as ps
    from paper_2604_00754_amd import binding as sa
    n, seed = 131072, 2 ** 64 - 3
    ref = ps.sample_perm(seed, 1, 1, 1, n)
    desc, perm = sample(1, 1, 1, 1, n, seed, 1)
    assert np.array_equal(perm.cpu().numpy(), ref)
    desc, perm = sample(1, 1, 1, 1, n, seed, 1, workspace=True)
    assert np.array_equal(perm.cpu().numpy(), ref)
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_CHECK_PERM), device=U.DEV, dtype=torch.uint8)
    sa.sa_check_perm(desc, perm, ws)  # raises unless every slice is a bijection


def test_sampled_permutation_feeds_the_attention_kernel():
    """The sampler's output is used as it is: sa_fwd with the device-sampled permutation against the
    oracle run with the oracle-sampled one."""
    from oracle import binding as orc
    from oracle import perm_sampler as ps
    from paper_2604_00754_amd import binding as sa
    B, H, n, d, w = 1, 2, 700, 64, 64
    wl, x = U.make_case(B, H, H, n, d, w, "bf16", 1, 2, seed=70)
    desc = sa.make_desc(B, H, H, n, d, w, perm_B=1, perm_H=2)
    perm = torch.empty((1, 2, n), device=U.DEV, dtype=torch.int32)
    sa.sa_sample_perm(desc, 99, 2, perm)
    Q, K, V = (U.to_dev(x[k], "bf16") for k in "QKV")
    Y = torch.empty_like(Q)
    sa.sa_fwd(desc, Q, K, V, perm, Y, None)
    torch.cuda.synchronize()
    Yr, _ = orc.sa_fwd(orc.desc(B, H, H, n, d, w, orc.WIN_SYM_CIRCULAR, 1, 1, 2), x["Q"], x["K"], x["V"],
                       ps.sample_perm(99, 2, 1, 2, n))
    U.assert_close(U.to_np64(Y), Yr, "bf16", "Y")


def test_sample_perm_rejects_bad_arguments():
    from paper_2604_00754_amd import binding as sa
    desc = sa.make_desc(1, 1, 1, 16, 64, 4)
    with pytest.raises(sa.SaError) as e:
        sa.sa_sample_perm(desc, 1, 0, None)
    assert e.value.status == sa.SA_ERR_NULL
    perm = torch.empty((1, 1, 16), device=U.DEV, dtype=torch.int32)
    with pytest.raises(sa.SaError) as e:
        sa.sa_sample_perm(desc, 1, -1, perm)
    assert e.value.status == sa.SA_ERR_SHAPE
    big = sa.make_desc(1, 1, 1, 4096, 64, 4)
    perm = torch.empty((1, 1, 4096), device=U.DEV, dtype=torch.int32)
    ws = torch.empty(sa.sa_workspace_bytes(big, sa.SA_OP_SAMPLE_PERM) - 1, device=U.DEV, dtype=torch.uint8)
    with pytest.raises(sa.SaError) as e:
        sa.sa_sample_perm(big, 1, 0, perm, ws)
    assert e.value.status == sa.SA_ERR_WORKSPACE
