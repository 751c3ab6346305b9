"""GPU parity of sa_decode_fwd (the full-cache decoding step of the inference setting, Sec. 4.2) against the
fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def run_decode(B, Hq, Hkv, n, d, length, dtype="bf16", seed=0, poison=True, scale=0.0):
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    print(f"case decode B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} len{length} {dtype} seed{seed} scale{scale}", flush=True)
    wl, x = U.make_case(B, Hq, Hkv, n, d, 2, dtype, seed=seed, identity=True)
    q = U.to_dev(np.ascontiguousarray(x["Q"][:, :, length - 1]), dtype)
    K, V = U.to_dev(x["K"], dtype), U.to_dev(x["V"], dtype)
    q64, k64, v64 = U.to_np64(q), U.to_np64(K), U.to_np64(V)
    if poison and length < n:          # rows past `length` are not part of the cache yet
        K[:, :, length:] = float("nan")
        V[:, :, length:] = float("nan")
    desc = sa.make_desc(B, Hq, Hkv, n, d, 2, dtype=sa.SA_BF16 if dtype == "bf16" else sa.SA_F32, scale=scale)
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_DECODE), dtype=torch.uint8, device=U.DEV)
    Y = torch.full((B, Hq, d), float("nan"), device=U.DEV, dtype=U.tdtype(dtype))
    L = torch.full((B, Hq), float("nan"), device=U.DEV, dtype=torch.float32)
    sa.sa_decode_fwd(desc, q, K, V, length, Y, L, ws)
    torch.cuda.synchronize()
    Yr, Lr = orc.decode_fwd(orc.desc(B, Hq, Hkv, n, d, 2, scale=scale), q64, k64, v64, length)
    U.assert_close(U.to_np64(Y), Yr, dtype, "decode Y")
    assert np.abs(L.cpu().numpy().astype(np.float64) - Lr).max() <= (1e-4 if dtype == "f32" else 1e-3)
    return Y, L


@pytest.mark.parametrize("B,Hq,Hkv,n,d,length", [
    (1, 4, 4, 300, 64, 300),      # one query head per KV head
    (2, 8, 4, 700, 128, 513),     # two, batch of two, cache partly filled
    (1, 8, 2, 1100, 128, 1100),   # four (the Qwen3-8B ratio)
    (1, 8, 1, 900, 64, 777),      # eight (the Qwen3-30B-A3B ratio)
    (1, 16, 2, 900, 128, 900),    # eight, head size 128
    (1, 6, 2, 500, 128, 499),     # three: one head per workgroup
    (1, 12, 1, 400, 64, 400),     # twelve: three sets of four
    (3, 4, 2, 4096, 64, 100),     # large capacity, short cache
])
def test_bf16_parity_group_sizes(B, Hq, Hkv, n, d, length):
    run_decode(B, Hq, Hkv, n, d, length)


@pytest.mark.parametrize("B,Hq,Hkv,n,d,length", [(1, 2, 2, 1024, 64, 1000), (2, 4, 1, 600, 128, 600),
                                                  (1, 8, 1, 333, 64, 333)])
def test_f32_parity(B, Hq, Hkv, n, d, length):
    run_decode(B, Hq, Hkv, n, d, length, dtype="f32")


@pytest.mark.parametrize("d", [64, 128])
def test_cache_lengths_around_load_and_chunk_edges(d):
    """Lengths around the rows of one wave-wide load (4 or 8), of one workgroup-wide load (16 or 32), of one
    unrolled iteration (64 or 128) and of a chunk (64 at this size)."""
    for length in (1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 193, 300):
        run_decode(1, 4, 1, 300, d, length, seed=length)


@pytest.mark.parametrize("B,Hq,Hkv,n,d,length", [
    (1, 4, 4, 1, 64, 1),          # a cache of one row
    (1, 8, 2, 65, 128, 65),       # second chunk holds a single row
    (2, 8, 8, 64, 128, 64),       # exactly one chunk
    (1, 32, 8, 2048, 128, 1025),  # chunks of 64 rows (few KV heads): 17 chunks, the last one ragged
    (64, 8, 8, 1024, 64, 1000),   # many sequences: chunks of 512 rows
])
def test_chunk_geometry_corner_cases(B, Hq, Hkv, n, d, length):
    run_decode(B, Hq, Hkv, n, d, length)


def test_softmax_scale_and_single_cached_row():
    from paper_2604_00754_amd import binding as sa
    run_decode(1, 8, 2, 257, 128, 200, scale=0.31)
    Y, L = run_decode(1, 4, 2, 64, 64, 1, seed=5)
    # one cached row: the output is that row, bit for bit
    wl, x = U.make_case(1, 4, 2, 64, 64, 2, "bf16", seed=5, identity=True)
    V = U.to_dev(x["V"], "bf16")
    assert torch.equal(Y[0], V[0, :, 0].repeat_interleave(2, dim=0))


def test_decode_continues_the_prompt_pass():
    """Hand-off of Sec. 4.2 on the GPU: the decoding step for the token at position len-1 over a cache of len
    rows returns the row that full causal attention over the prompt (one-sided window with w >= n) produces for
    that token, up to the rounding of the two bf16 outputs."""
    from paper_2604_00754_amd import binding as sa
    B, Hq, Hkv, n, d = 1, 8, 2, 640, 128
    wl, x = U.make_case(B, Hq, Hkv, n, d, n, "bf16", seed=3, identity=True)
    Q, K, V = (U.to_dev(x[k], "bf16") for k in "QKV")
    full = sa.make_desc(B, Hq, Hkv, n, d, n, sa.SA_WIN_ONE_SIDED, 1)
    Yp = torch.empty_like(Q)
    Lp = torch.empty((B, Hq, n), device=U.DEV, dtype=torch.float32)
    sa.swa_fwd(full, Q, K, V, Yp, Lp)
    ws = torch.empty(sa.sa_workspace_bytes(full, sa.SA_OP_DECODE), dtype=torch.uint8, device=U.DEV)
    for length in (1, 77, 640):
        Y = torch.empty((B, Hq, d), device=U.DEV, dtype=torch.bfloat16)
        L = torch.empty((B, Hq), device=U.DEV, dtype=torch.float32)
        sa.sa_decode_fwd(full, Q[:, :, length - 1].contiguous(), K, V, length, Y, L, ws)
        torch.cuda.synchronize()
        assert (Y.float() - Yp[:, :, length - 1].float()).abs().max().item() <= 2e-2
        # the prefill's row sum is taken from the bf16-rounded probabilities that build its output (|dLSE| <= 2^-9
        # plus the exp/log error), the decoding step sums in fp32: the two agree to the bf16 LSE bar
        assert (L - Lp[:, :, length - 1]).abs().max().item() <= 4e-3


@pytest.mark.parametrize("B,Hq,Hkv,n,d,lens", [
    (4, 8, 2, 1500, 128, [1500, 1, 700, 513]),
    (3, 8, 1, 900, 64, [64, 65, 900]),
    (5, 4, 4, 2100, 128, [2100, 2099, 33, 1024, 1025]),
    (2, 6, 2, 800, 128, [5, 300]),          # max_len below the capacity
])
def test_sequences_of_different_lengths(B, Hq, Hkv, n, d, lens):
    """sa_decode_fwd_varlen: every sequence of the batch against the oracle run on that sequence alone with its own
    length; rows beyond a sequence's length are NaN."""
    from oracle import binding as orc
    from paper_2604_00754_amd import binding as sa
    print(f"case decode varlen B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} lens{lens}", flush=True)
    wl, x = U.make_case(B, Hq, Hkv, n, d, 2, "bf16", seed=7, identity=True)
    q = U.to_dev(np.ascontiguousarray(x["Q"][:, :, 0]), "bf16")
    K, V = U.to_dev(x["K"], "bf16"), U.to_dev(x["V"], "bf16")
    q64, k64, v64 = U.to_np64(q), U.to_np64(K), U.to_np64(V)
    for b, ln in enumerate(lens):
        K[b, :, ln:] = float("nan")
        V[b, :, ln:] = float("nan")
    desc = sa.make_desc(B, Hq, Hkv, n, d, 2)
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_DECODE), dtype=torch.uint8, device=U.DEV)
    ws.fill_(255)   # NaN patterns: every partial result the merge reads must have been written
    Y = torch.full((B, Hq, d), float("nan"), device=U.DEV, dtype=torch.bfloat16)
    L = torch.full((B, Hq), float("nan"), device=U.DEV, dtype=torch.float32)
    lens_dev = torch.tensor(lens, device=U.DEV, dtype=torch.int32)
    sa.sa_decode_fwd_varlen(desc, q, K, V, lens_dev, max(lens), Y, L, ws)
    torch.cuda.synchronize()
    for b, ln in enumerate(lens):
        Yr, Lr = orc.decode_fwd(orc.desc(1, Hq, Hkv, n, d, 2), q64[b:b + 1], k64[b:b + 1], v64[b:b + 1], ln)
        U.assert_close(U.to_np64(Y[b:b + 1]), Yr, "bf16", f"decode Y, sequence {b}")
        assert np.abs(L[b:b + 1].cpu().numpy().astype(np.float64) - Lr).max() <= 1e-3
    # out-of-range entries are clamped to 1..max_len instead of reading outside the cache
    bad = torch.tensor([0] + [10 ** 9] * (B - 1), device=U.DEV, dtype=torch.int32)
    K2, V2 = U.to_dev(x["K"], "bf16"), U.to_dev(x["V"], "bf16")
    Y2 = torch.empty_like(Y)
    sa.sa_decode_fwd_varlen(desc, q, K2, V2, bad, max(lens), Y2, None, ws)
    torch.cuda.synchronize()
    Yr, _ = orc.decode_fwd(orc.desc(1, Hq, Hkv, n, d, 2), q64[:1], k64[:1], v64[:1], 1)
    U.assert_close(U.to_np64(Y2[:1]), Yr, "bf16", "clamped to one row")
    Yr, _ = orc.decode_fwd(orc.desc(1, Hq, Hkv, n, d, 2), q64[1:2], k64[1:2], v64[1:2], max(lens))
    U.assert_close(U.to_np64(Y2[1:2]), Yr, "bf16", "clamped to max_len")


@pytest.mark.parametrize("Hq,Hkv,n,length", [(32, 8, 32768, 32768), (32, 8, 32768, 30001), (32, 4, 131072, 131072)])
def test_full_size_caches(Hq, Hkv, n, length):
    """The cache of the headline prefill shape (Qwen3-8B heads, 32K rows) and of the long one (32/4 heads, 128K
    rows), every output checked against the oracle."""
    run_decode(1, Hq, Hkv, n, 128, length, poison=False)
