"""The calls of the inference sequence of Sec. 4.2 (rotate K, stochastic-attention prefill with the Q rotation
fused, full-cache decoding step) and of a training step (forward, backward) only enqueue kernels on the caller's
stream, so they can be recorded into a HIP graph.  Each graph is replayed several times, with eager work and
synchronisations in between and fresh inputs before each replay, and every replay must reproduce the eager
result bit for bit."""
import numpy as np
import pytest
import torch

from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def fresh(shape, seed):
    g = torch.Generator(device=U.DEV)
    g.manual_seed(seed)
    return torch.randn(shape, device=U.DEV, dtype=torch.float32, generator=g).to(torch.bfloat16)


def test_prefill_and_decode_replay_from_a_graph():
    from paper_2604_00754_amd import binding as sa, synth
    B, Hq, Hkv, n, d, w = 1, 8, 2, 1536, 128, 128
    print(f"case graph prefill+decode B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} w{w}", flush=True)
    desc = sa.make_desc(B, Hq, Hkv, n, d, w)
    perm = torch.from_numpy(synth.permutations(1, 1, n, seed=1)).to(U.DEV)
    table = torch.empty((n, d // 2, 2), device=U.DEV, dtype=torch.float32)
    sa.sa_rope_table(n, d, 1e6, 0, table)
    Q, K, V = fresh((B, Hq, n, d), 1), fresh((B, Hkv, n, d), 2), fresh((B, Hkv, n, d), 3)
    q1 = fresh((B, Hq, d), 4)
    Kr, Y = torch.empty_like(K), torch.empty_like(Q)
    L = torch.empty((B, Hq, n), device=U.DEV, dtype=torch.float32)
    Yd = torch.empty((B, Hq, d), device=U.DEV, dtype=torch.bfloat16)
    Ld = torch.empty((B, Hq), device=U.DEV, dtype=torch.float32)
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_DECODE), device=U.DEV, dtype=torch.uint8)

    def sequence():
        sa.sa_rope(desc, None, K, table, None, Kr)
        sa.sa_fwd_rope(desc, Q, Kr, V, perm, table, Y, L)
        sa.sa_decode_fwd(desc, q1, Kr, V, n - 5, Yd, Ld, ws)

    sequence()                      # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sequence()
    for rep in range(4):
        for t, seed in ((Q, 10), (K, 20), (V, 30), (q1, 40)):
            t.copy_(fresh(t.shape, seed + rep))
        sequence()                  # eager reference on the same buffers
        torch.cuda.synchronize()
        want = [x.clone() for x in (Y, L, Yd, Ld)]
        for x in (Kr, Y, L, Yd, Ld):
            x.fill_(float("nan"))
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, name in zip((Y, L, Yd, Ld), want, ("Y", "LSE", "Y_decode", "LSE_decode")):
            assert torch.equal(got, ref), f"replay {rep}: {name} differs from the eager call"


def test_training_step_replays_from_a_graph():
    from paper_2604_00754_amd import binding as sa, synth
    B, H, n, d, w = 2, 4, 1024, 64, 64
    print(f"case graph fwd+bwd B{B} H{H} n{n} d{d} w{w}", flush=True)
    desc = sa.make_desc(B, H, H, n, d, w)
    perm = torch.from_numpy(synth.permutations(1, 1, n, seed=2)).to(U.DEV)
    Q, K, V, dY = (fresh((B, H, n, d), s) for s in (1, 2, 3, 4))
    Y, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
    L = torch.empty((B, H, n), device=U.DEV, dtype=torch.float32)
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_BWD), device=U.DEV, dtype=torch.uint8)

    def step():
        sa.sa_fwd(desc, Q, K, V, perm, Y, L)
        sa.sa_bwd(desc, None, Q, K, V, perm, None, None, Y, None, L, None, dY, dQ, dK, dV, None, None, ws)

    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t, seed in ((Q, 10), (K, 20), (V, 30), (dY, 40)):
            t.copy_(fresh(t.shape, seed + rep))
        step()
        torch.cuda.synchronize()
        want = [x.clone() for x in (Y, L, dQ, dK, dV)]
        for x in (Y, L, dQ, dK, dV):
            x.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, name in zip((Y, L, dQ, dK, dV), want, ("Y", "LSE", "dQ", "dK", "dV")):
            assert torch.equal(got, ref), f"replay {rep}: {name} differs from the eager call"


def test_training_step_with_fused_rotations_replays_from_a_graph():
    """rotate K, forward with the Q rotation fused, backward with the Q / dQ / dK rotations fused: the workspace of
    sa_bwd_rope (row sums and the rotated query rows the dQ kernel leaves for the dK/dV kernel) is rewritten by
    every call, so a replay on fresh inputs must reproduce the eager step bit for bit."""
    from paper_2604_00754_amd import binding as sa, synth
    B, Hq, Hkv, n, d, w = 1, 8, 2, 1280, 128, 128
    print(f"case graph rope fwd+bwd B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} w{w}", flush=True)
    desc = sa.make_desc(B, Hq, Hkv, n, d, w)
    perm = torch.from_numpy(synth.permutations(1, 1, n, seed=3)).to(U.DEV)
    table = torch.empty((n, d // 2, 2), device=U.DEV, dtype=torch.float32)
    sa.sa_rope_table(n, d, 1e6, 0, table)
    Q, dY = fresh((B, Hq, n, d), 1), fresh((B, Hq, n, d), 4)
    K, V = fresh((B, Hkv, n, d), 2), fresh((B, Hkv, n, d), 3)
    Kr, dK, dV = torch.empty_like(K), torch.empty_like(K), torch.empty_like(K)
    Y, dQ = torch.empty_like(Q), torch.empty_like(Q)
    L = torch.empty((B, Hq, n), device=U.DEV, dtype=torch.float32)
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_BWD_ROPE), device=U.DEV, dtype=torch.uint8)

    def step():
        sa.sa_rope(desc, None, K, table, None, Kr)
        sa.sa_fwd_rope(desc, Q, Kr, V, perm, table, Y, L)
        sa.sa_bwd_rope(desc, Q, Kr, V, perm, table, Y, L, dY, dQ, dK, dV, ws, dk_unrotated=1)

    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t, seed in ((Q, 10), (K, 20), (V, 30), (dY, 40)):
            t.copy_(fresh(t.shape, seed + rep))
        step()
        torch.cuda.synchronize()
        want = [x.clone() for x in (Y, L, dQ, dK, dV)]
        for x in (Kr, Y, L, dQ, dK, dV):
            x.fill_(float("nan"))
        ws.fill_(255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, name in zip((Y, L, dQ, dK, dV), want, ("Y", "LSE", "dQ", "dK", "dV")):
            assert torch.equal(got, ref), f"replay {rep}: {name} differs from the eager call"
