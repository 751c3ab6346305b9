"""sa_decode_fwd_static, the entry point for callers that cannot allocate: its output against sa_decode_fwd's
(the same kernels with a caller-owned workspace) and against the fp64 oracle, on two calls in a row, the second
with a smaller input, so that the second call runs on a buffer that still holds the first call's partial results."""
import numpy as np
import pytest
import torch

from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def run_pair(B, Hq, Hkv, n, d, length, seed):
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    print(f"case decode_static B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} len{length}", flush=True)
    g = torch.Generator(device=U.DEV)
    g.manual_seed(seed)
    q = torch.randn((B, Hq, d), device=U.DEV, generator=g).to(torch.bfloat16)
    K = torch.randn((B, Hkv, n, d), device=U.DEV, generator=g).to(torch.bfloat16)
    V = torch.randn((B, Hkv, n, d), device=U.DEV, generator=g).to(torch.bfloat16)
    desc = sa.make_desc(B, Hq, Hkv, n, d, 2)
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_DECODE), device=U.DEV, dtype=torch.uint8)
    Y0 = torch.full_like(q, float("nan"))
    L0 = torch.full((B, Hq), float("nan"), device=U.DEV, dtype=torch.float32)
    sa.sa_decode_fwd(desc, q, K, V, length, Y0, L0, ws)
    Y1, L1 = torch.full_like(Y0, float("nan")), torch.full_like(L0, float("nan"))
    sa.sa_decode_fwd_static(desc, q, K, V, length, Y1, L1)
    torch.cuda.synchronize()
    # same kernels, same launch geometry: bit for bit
    assert torch.equal(Y0.view(torch.int16), Y1.view(torch.int16))
    assert torch.equal(L0, L1)
    Yr, Lr = orc.decode_fwd(orc.desc(B, Hq, Hkv, n, d, 2), U.to_np64(q), U.to_np64(K), U.to_np64(V), length)
    U.assert_close(U.to_np64(Y1), Yr, "bf16", "decode_static Y")
    assert np.abs(L1.cpu().numpy().astype(np.float64) - Lr).max() <= 4e-3


def test_static_decode_two_calls_second_smaller():
    run_pair(2, 32, 8, 8192, 128, 8000, seed=5)    # 16 chunks per head: fills 2*32*16 partial results
    run_pair(1, 8, 2, 1000, 64, 333, seed=6)       # smaller: fewer heads, fewer chunks, other head size
    run_pair(2, 32, 8, 8192, 128, 700, seed=7)     # the first shape again with a short sequence


def test_static_decode_rejects_beyond_its_buffer():
    from paper_2604_00754_amd import binding as sa
    big = sa.make_desc(16, 32, 8, 131072, 128, 2)
    x = torch.zeros(16, device=U.DEV, dtype=torch.bfloat16)
    with pytest.raises(sa.SaError) as e:
        sa.sa_decode_fwd_static(big, x, x, x, 16, x, None)
    assert e.value.status == sa.SA_ERR_STATIC_LIMIT
