#!/usr/bin/env python3
"""Benchmark of the Stochastic Attention hot path on one MI355X.

A step is one sa_fwd call (gather through the permutation, windowed attention in permuted order,
scatter back) on the Qwen3-8B-shaped prefill layer: B=1, 32 query heads, 8 KV heads, d=128,
n=32768, w=512, bf16, one permutation shared by the heads, circular symmetric window in slot space
with the causal constraint on original positions.  Inputs are synthetic N(0,1) tensors already
resident in HBM.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "SA fwd(+bwd) tokens/s and TFLOP/s (% bf16 MFMA peak) at n=32K, w=512"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
CSRC = os.path.join(ROOT, "paper_2604_00754_amd", "csrc")


def measured_traffic(op, workload):
    """HBM bytes per call of `op` on `workload` as the hardware counters saw them: taken from the `traffic-record:`
    line of a summary under profiles/ (two rocprofv3 --pmc runs, FETCH_SIZE and WRITE_SIZE, each scaled by what the
    same counter reads for a 1 GiB copy).  The record names the kernel sources it was taken with and their
    SHA-256; if the sources in this tree differ, the figure belongs to other kernels and None is returned."""
    import glob
    import hashlib
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        for line in open(path):
            if not line.startswith("traffic-record:"):
                continue
            rec = dict(kv.split("=", 1) for kv in line.split()[1:])
            if rec.get("op") != op or rec.get("workload") != workload:
                continue
            h = hashlib.sha256()
            for name in rec["sources"].split(","):
                with open(os.path.join(CSRC, name), "rb") as f:
                    h.update(f.read())
            if h.hexdigest() != rec["sha256"]:
                return None, f"{os.path.basename(path)}: kernel sources changed since the counters were read"
            nbytes = (float(rec["fetch_kib"]) * float(rec["fetch_scale"]) +
                      float(rec["write_kib"]) * float(rec["write_scale"])) * 1024.0
            return nbytes, f"{os.path.basename(path)} (commit {rec.get('commit', '?')})"
    return None, "no counter run on record for this call"


def band_slots(n, w, window):
    """Slots inside one query's window (the band the kernel must contract over)."""
    if window == 2:
        return None  # one-sided: depends on the row, handled by the caller
    h = (w - 1) // 2
    return min(2 * h + 1, n)


def time_op(fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    samples = [a.elapsed_time(b) for a, b in ev]
    time_op.last_samples_ms = samples
    return wall, float(np.mean(samples))


def time_side(fn, steps, warmup):
    """Side measurements: the median of the per-call HIP-event times (a single slow call -- a clock ramp, a first
    touch of a workspace -- would otherwise dominate the mean of a handful of calls).  Same return shape as
    time_op."""
    wall, _ = time_op(fn, steps, warmup)
    return wall, float(np.median(time_op.last_samples_ms))


def time_pair(fn_a, fn_b, steps, warmup):
    """Two variants of one call, timed alternately (a, b, a, b, ...) so that a drift of the clocks during the
    measurement falls on both alike; the median per-call HIP-event time of each."""
    for _ in range(warmup):
        fn_a()
        fn_b()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for a0, a1, b0, b1 in ev:
        a0.record()
        fn_a()
        a1.record()
        b0.record()
        fn_b()
        b1.record()
    torch.cuda.synchronize()
    return (float(np.median([e[0].elapsed_time(e[1]) for e in ev])),
            float(np.median([e[2].elapsed_time(e[3]) for e in ev])))


def executed_flop(n, w, d, B, Hq, BM=128, BN=64):
    """Flop of the matrix instructions the forward kernel issues at this shape (symmetric circular
    window): per wave (32 query slots) every 32-key block of the workgroup's tiles that any of its
    queries can see, each costing 2 * (d/16) MFMAs of 32x32x16.  BM = query slots of a workgroup (128, or
    64 / 32 when it takes 2 / 4 query heads of a KV group over the same slots)."""
    h = (w - 1) // 2
    L, R = min(h, (n - 1) // 2), 0
    R = min(h, n - 1 - L)
    per_block = 2 * (d // 16) * 2 * 32 * 32 * 16
    total_blocks = 0
    for p0 in range(0, n, BM):
        q_last = min(p0 + BM - 1, n - 1)
        t_lo, t_hi = p0 - L, q_last + R
        ntiles = (t_hi - t_lo + BN) // BN
        for wave in range(BM // 32):
            s_w0 = p0 + 32 * wave
            if s_w0 >= n:
                continue  # such a wave still runs, on clamped rows; not counted
            for blk in range((BN // 32) * ntiles):
                tb0 = t_lo + 32 * blk
                dmax, dmin = tb0 + 31 - s_w0, tb0 - (s_w0 + 31)
                if not (dmax < -L or dmin > R) and tb0 <= t_hi:
                    total_blocks += 1
    return float(total_blocks) * per_block * B * Hq


def heads_per_workgroup(wl):
    """Query heads of a KV group that one workgroup of the forward kernel takes (over the same slots) when
    they share a permutation: 4, 2 or 1 by group size; 1 with per-head permutations."""
    g = wl.Hq // wl.Hkv
    if wl.perm_H != 1:
        return 1
    return 4 if g % 4 == 0 else (2 if g % 2 == 0 else 1)


def cpu_baseline(wl, Q, K, V, perm, rows_per_head):
    """The fp64 oracle, as it stands, on a row sample of the same workload."""
    from oracle import binding as orc
    from paper_2604_00754_amd import synth
    c = orc.desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, orc.WIN_SYM_CIRCULAR, 1, 1, 1)
    rows = synth.sample_rows(wl.B, wl.Hq, wl.n, rows_per_head, seed=7)
    Q64, K64, V64 = (x.to(torch.float32).cpu().numpy().astype(np.float64) for x in (Q, K, V))
    t0 = time.perf_counter()
    Y, _ = orc.sa_fwd_rows(c, Q64, K64, V64, perm.cpu().numpy(), rows)
    dt = time.perf_counter() - t0
    # pairs the mask leaves visible (the permutation is shared by the heads: count one head)
    c1 = orc.desc(1, 1, 1, wl.n, wl.d, wl.w, orc.WIN_SYM_CIRCULAR, 1, 1, 1)
    visible_pairs = int(orc.visible_count(c1, perm.cpu().numpy()).sum())
    tokens = rows.shape[0] / wl.Hq  # one token = one position across all query heads
    return {"value": tokens / dt, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "useful_flop": 4.0 * wl.d * visible_pairs * wl.B * wl.Hq,
            "sample": f"{rows_per_head} of {wl.n} query rows per head, all {wl.Hq} heads "
                      f"({rows.shape[0]} rows, {dt:.1f} s)"}, rows, Y


def training_ops(sa, synth, dev, reps):
    """Side measurements (not the headline): the pre-training shapes, forward and backward.
    B=4, H=16, n=8192, d=64, w=256: ungated SA fwd+bwd and gated SA+SWA fwd+bwd."""
    wl = synth.WORKLOADS["pretrain_fwdbwd_8k"]
    B, H, n, d, w = wl.B, wl.Hq, wl.n, wl.d, wl.w
    g = torch.Generator(device=dev)
    g.manual_seed(synth.BASE_SEED + 1)
    rn = lambda shape, dt=torch.bfloat16: torch.randn(shape, device=dev, dtype=torch.float32, generator=g).to(dt)
    Q, K, V, dY = (rn((B, H, n, d)) for _ in range(4))
    ga, gl = rn((B, H, n), torch.float32), rn((B, H, n), torch.float32)
    perm = torch.from_numpy(synth.permutations(1, 1, n)).to(dev)
    dsa = sa.make_desc(B, H, H, n, d, w, sa.SA_WIN_SYM_CIRCULAR, 1, sa.SA_BF16, 0.0, 1, 1)
    dswa = sa.make_desc(B, H, H, n, d, w, sa.SA_WIN_ONE_SIDED, 1, sa.SA_BF16, 0.0, 1, 1)
    Y, Ysa, Yswa, dQ, dK, dV = (torch.empty_like(Q) for _ in range(6))
    Lsa = torch.empty((B, H, n), device=dev, dtype=torch.float32)
    Lswa, dga, dgl = torch.empty_like(Lsa), torch.empty_like(ga), torch.empty_like(gl)
    wsf = torch.empty(sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_FWD), device=dev, dtype=torch.uint8)
    wsb = torch.empty(sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_BWD), device=dev, dtype=torch.uint8)
    _, t_fwd = time_side(lambda: sa.sa_fwd(dsa, Q, K, V, perm, Ysa, Lsa), reps, 2)
    _, t_bwd = time_side(lambda: sa.sa_bwd(dsa, None, Q, K, V, perm, None, None, Ysa, None, Lsa, None, dY,
                                         dQ, dK, dV, None, None, wsb), reps, 2)
    _, t_gfwd = time_side(lambda: sa.gated_sa_swa_fwd(dsa, dswa, Q, K, V, perm, ga, gl, Y, Ysa, Yswa, Lsa, Lswa,
                                                    wsf), reps, 2)
    _, t_gbwd = time_side(lambda: sa.sa_bwd(dsa, dswa, Q, K, V, perm, ga, gl, Ysa, Yswa, Lsa, Lswa, dY,
                                          dQ, dK, dV, dga, dgl, wsb), reps, 2)
    # the gate projections of the paper's layer (Eq. 6 + Eq. 5) on the two branch outputs, d_model = H*d
    dm = H * d
    Wsa, Wswa = (rn((dm, dm), torch.float32).mul_(dm ** -0.5).to(torch.bfloat16) for _ in range(2))
    Gsa, Gswa, dYsa, dYswa = (torch.empty_like(Q) for _ in range(4))
    dWsa, dWswa = torch.empty_like(Wsa), torch.empty_like(Wswa)
    wsg = torch.empty(sa.sa_workspace_bytes(dsa, sa.SA_OP_GATE_PROJ_BWD), device=dev, dtype=torch.uint8)
    # training form and inference form (the gate values are not kept: two of the three output tensors are not
    # written), timed alternately
    t_gp, t_gpi = time_pair(lambda: sa.sa_gate_proj_fwd(dsa, Ysa, Yswa, Wsa, Wswa, Y, Gsa, Gswa),
                            lambda: sa.sa_gate_proj_fwd(dsa, Ysa, Yswa, Wsa, Wswa, Y, None, None), reps, 2)
    _, t_gpb = time_side(lambda: sa.sa_gate_proj_bwd(dsa, Ysa, Yswa, Wsa, Wswa, Gsa, Gswa, dY, dYsa, dYswa,
                                                   dWsa, dWswa, wsg), reps, 2)
    # the whole layer of Alg. 2 in one call each way (both branches + gate projections)
    wsd = torch.empty(sa.sa_workspace_bytes(dsa, sa.SA_OP_DUAL_PATH_BWD), device=dev, dtype=torch.uint8)
    _, t_dpf = time_side(lambda: sa.sa_dual_path_fwd(dsa, dswa, Q, K, V, perm, Wsa, Wswa, Y, Ysa, Yswa, Gsa, Gswa,
                                                   Lsa, Lswa), reps, 2)
    _, t_dpb = time_side(lambda: sa.sa_dual_path_bwd(dsa, dswa, Q, K, V, perm, Wsa, Wswa, Ysa, Yswa, Gsa, Gswa,
                                                   Lsa, Lswa, dY, dQ, dK, dV, dWsa, dWswa, wsd), reps, 2)
    del Gsa, Gswa, dYsa, dYswa, wsg, wsd
    flop_gp = 2 * 2.0 * B * n * dm * dm
    W = band_slots(n, w, 0)
    flop_fb = 14.0 * n * W * d * B * H  # forward 4, backward 10 per (query, in-window slot, d)
    return {"pretrain_8k": {
        "gate_proj_fwd_ms": t_gp, "gate_proj_fwd_tflops": flop_gp / (t_gp * 1e-3) / 1e12,
        "gate_proj_fwd_frac_mfma_peak": flop_gp / (t_gp * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "gate_proj_fwd_no_gate_outputs_ms": t_gpi,
        "gate_proj_fwd_no_gate_outputs_tflops": flop_gp / (t_gpi * 1e-3) / 1e12,
        "gate_proj_bwd_ms": t_gpb, "gate_proj_bwd_tflops": 2 * flop_gp / (t_gpb * 1e-3) / 1e12,
        "shape": "B4 H16 n8192 d64 w256 bf16",
        "sa_fwd_ms": t_fwd, "sa_bwd_ms": t_bwd,
        "sa_fwdbwd_tokens_per_s": B * n / ((t_fwd + t_bwd) * 1e-3),
        "sa_fwdbwd_band_tflops": flop_fb / ((t_fwd + t_bwd) * 1e-3) / 1e12,
        "gated_fwd_ms": t_gfwd, "gated_bwd_ms": t_gbwd,
        "gated_fwdbwd_tokens_per_s": B * n / ((t_gfwd + t_gbwd) * 1e-3),
        "dual_path_layer_fwd_ms": t_dpf, "dual_path_layer_bwd_ms": t_dpb,
        "dual_path_layer_fwdbwd_tokens_per_s": B * n / ((t_dpf + t_dpb) * 1e-3)}}


def long_prefill_ops(sa, synth, dev, reps):
    """Side measurement: the long-prefill shape (B=1, 32 query / 4 KV heads, d=128, n=131072, w=1024),
    SA forward and plain SWA forward side by side."""
    wl = synth.WORKLOADS["qwen3_30b_prefill_128k"]
    g = torch.Generator(device=dev)
    g.manual_seed(synth.BASE_SEED + 2)
    rn = lambda shape: torch.randn(shape, device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16)
    Q, K, V = rn((wl.B, wl.Hq, wl.n, wl.d)), rn((wl.B, wl.Hkv, wl.n, wl.d)), rn((wl.B, wl.Hkv, wl.n, wl.d))
    perm = torch.from_numpy(synth.permutations(1, 1, wl.n)).to(dev)
    Y = torch.empty_like(Q)
    dsa = sa.make_desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, sa.SA_WIN_SYM_CIRCULAR, 1, sa.SA_BF16, 0.0, 1, 1)
    dswa = sa.make_desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, sa.SA_WIN_ONE_SIDED, 1, sa.SA_BF16, 0.0, 1, 1)
    _, t_sa = time_side(lambda: sa.sa_fwd(dsa, Q, K, V, perm, Y, None), reps, 1)
    _, t_swa = time_side(lambda: sa.swa_fwd(dswa, Q, K, V, Y, None), reps, 1)
    flop_sa = 4.0 * wl.n * band_slots(wl.n, wl.w, 0) * wl.d * wl.B * wl.Hq
    return {"long_prefill_128k": {
        "shape": "B1 Hq32 Hkv4 n131072 d128 w1024 bf16",
        "sa_fwd_ms": t_sa, "sa_fwd_tokens_per_s": wl.B * wl.n / (t_sa * 1e-3),
        "sa_fwd_band_tflops": flop_sa / (t_sa * 1e-3) / 1e12,
        "swa_fwd_ms": t_swa, "swa_fwd_tokens_per_s": wl.B * wl.n / (t_swa * 1e-3)}}


def backward_setup(sa, synth, dev, name):
    """Tensors and the call for sa_bwd (ungated, one permutation shared by the heads) on a named workload."""
    wl = synth.WORKLOADS[name]
    g = torch.Generator(device=dev)
    g.manual_seed(synth.BASE_SEED + 3)
    rn = lambda shape: torch.randn(shape, device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16)
    Q, dY = rn((wl.B, wl.Hq, wl.n, wl.d)), rn((wl.B, wl.Hq, wl.n, wl.d))
    K, V = rn((wl.B, wl.Hkv, wl.n, wl.d)), rn((wl.B, wl.Hkv, wl.n, wl.d))
    perm = torch.from_numpy(synth.permutations(1, 1, wl.n)).to(dev)
    desc = sa.make_desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, sa.SA_WIN_SYM_CIRCULAR, 1, sa.SA_BF16, 0.0, 1, 1)
    Y, dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    L = torch.empty((wl.B, wl.Hq, wl.n), device=dev, dtype=torch.float32)
    ws = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_BWD), device=dev, dtype=torch.uint8)
    sa.sa_fwd(desc, Q, K, V, perm, Y, L)
    keep = (Q, K, V, dY, perm, Y, dQ, dK, dV, L, ws)

    def call():
        sa.sa_bwd(desc, None, Q, K, V, perm, None, None, Y, None, L, None, dY, dQ, dK, dV, None, None, ws)
    return wl, call, keep


def backward_roofline(sa, synth, dev, steps, warmup):
    """The second half of the metric: sa_bwd (dQ kernel, which also forms the row sums D, then dK/dV kernel) on the pre-training
    shape B=4, H=16, n=8192, d=64, w=256, against both roofs.  Algorithmic flop: 5 contractions over the window
    band, 10 n W d per (b, h); algorithmic bytes: Q, K, V, Y, dY, LSE and the index tensor in, dQ, dK, dV out."""
    wl, call, keep = backward_setup(sa, synth, dev, "pretrain_fwdbwd_8k")
    _, mean_ms = time_op(call, steps, warmup)
    samples = list(time_op.last_samples_ms)
    W = band_slots(wl.n, wl.w, 0)
    flop = 10.0 * wl.n * W * wl.d * wl.B * wl.Hq
    e = 2
    nbytes = wl.B * wl.n * wl.d * e * (5 * wl.Hq + 3 * wl.Hkv) + wl.B * wl.Hq * wl.n * 4 + wl.n * 4
    tflops, gbs = flop / (mean_ms * 1e-3) / 1e12, nbytes / (mean_ms * 1e-3) / 1e9
    traffic, source = measured_traffic("sa_bwd", "pretrain_fwdbwd_8k")
    return {"op": "sa_bwd", "workload": "pretrain_fwdbwd_8k", "shape": "B4 H16 n8192 d64 w256 bf16",
            "kernels": ["bwd_dq_mfma_bf16_kernel<64, 2>", "bwd_dkv_mfma_bf16_kernel<64, 2>"],
            "dominant_kernel": "bwd_dkv_mfma_bf16_kernel<64, 2>",
            "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
            "algorithmic_bytes": nbytes, "traffic": traffic, "traffic_source": source,
            "mfma": {"achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tflops / PEAK_BF16_TFLOPS,
                     "algorithmic_flop": flop},
            "avg_call_ms": mean_ms, "median_call_ms": float(np.median(samples)), "min_call_ms": float(np.min(samples)),
            "note": "one sa_bwd call = two kernels; the nearer roof at this shape is HBM (frac), the MFMA figure beside it"}


def table3_sweep(sa, synth, dev):
    """Sec. 4.3 / Table 3 on this GPU: attention forward + backward in isolation, B=16, H=16, d=64,
    w=256, bf16, n = 2K ... 32K: single-path SA, plain causal SWA, gated SA+SWA, and full causal
    attention run through the same kernels with a window that covers the whole ring."""
    B, H, d, w = 16, 16, 64, 256
    out = []
    for n in (2048, 4096, 8192, 16384, 32768):
        g = torch.Generator(device=dev)
        g.manual_seed(synth.BASE_SEED + n)
        rn = lambda shape, dt=torch.bfloat16: torch.randn(shape, device=dev, dtype=torch.float32, generator=g).to(dt)
        Q, K, V, dY = (rn((B, H, n, d)) for _ in range(4))
        ga, gl = rn((B, H, n), torch.float32), rn((B, H, n), torch.float32)
        perm = torch.from_numpy(synth.permutations(1, 1, n)).to(dev)
        Y, Ysa, Yswa, dQ, dK, dV = (torch.empty_like(Q) for _ in range(6))
        Lsa = torch.empty((B, H, n), device=dev, dtype=torch.float32)
        Lswa, dga, dgl = torch.empty_like(Lsa), torch.empty_like(ga), torch.empty_like(gl)
        dsa = sa.make_desc(B, H, H, n, d, w, sa.SA_WIN_SYM_CIRCULAR, 1, sa.SA_BF16, 0.0, 1, 1)
        dswa = sa.make_desc(B, H, H, n, d, w, sa.SA_WIN_ONE_SIDED, 1, sa.SA_BF16, 0.0, 1, 1)
        dfull = sa.make_desc(B, H, H, n, d, n, sa.SA_WIN_ONE_SIDED, 1, sa.SA_BF16, 0.0, 1, 1)
        wsf = torch.empty(sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_FWD), device=dev, dtype=torch.uint8)
        wsb = torch.empty(sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_BWD), device=dev, dtype=torch.uint8)

        def fwd_bwd(desc, pm):
            sa.sa_fwd(desc, Q, K, V, pm, Ysa, Lsa)
            sa.sa_bwd(desc, None, Q, K, V, pm, None, None, Ysa, None, Lsa, None, dY, dQ, dK, dV, None, None, wsb)

        def gated():
            sa.gated_sa_swa_fwd(dsa, dswa, Q, K, V, perm, ga, gl, Y, Ysa, Yswa, Lsa, Lswa, wsf)
            sa.sa_bwd(dsa, dswa, Q, K, V, perm, ga, gl, Ysa, Yswa, Lsa, Lswa, dY, dQ, dK, dV, dga, dgl, wsb)

        reps = 10 if n <= 8192 else 5
        _, t_sa = time_side(lambda: fwd_bwd(dsa, perm), reps, 2)
        _, t_swa = time_side(lambda: fwd_bwd(dswa, None), reps, 2)
        _, t_g = time_side(gated, reps, 2)
        _, t_full = time_side(lambda: fwd_bwd(dfull, None), 2 if n >= 16384 else 4, 1)
        out.append({"n": n, "sa_fwdbwd_ms": t_sa, "swa_fwdbwd_ms": t_swa, "gated_sa_swa_fwdbwd_ms": t_g,
                    "full_causal_fwdbwd_ms": t_full, "full_over_sa": t_full / t_sa, "gated_over_sa": t_g / t_sa})
        print(f"table3 n={n}: SA {t_sa:.3f} ms  SWA {t_swa:.3f}  gated {t_g:.3f}  full {t_full:.2f}  "
              f"full/SA {t_full / t_sa:.1f}x", file=sys.stderr, flush=True)
        del Q, K, V, dY, Y, Ysa, Yswa, dQ, dK, dV, wsf, wsb
        torch.cuda.empty_cache()
    return {"table3_sweep": {"shape": "B16 H16 d64 w256 bf16, attention forward+backward", "rows": out}}


def profile_side_op(sa, synth, dev, args):
    """One entry point other than the headline step, called --steps times: for kernel traces and counter runs."""
    copy_src = copy_dst = None
    if args.calibrate_copy:
        copy_src = torch.zeros(256 * 1024 * 1024, device=dev, dtype=torch.float32)  # 1 GiB
        copy_dst = torch.empty_like(copy_src)
    if args.profile_op == "gated_fwd":
        wl = synth.WORKLOADS["pretrain_fwdbwd_8k"]
        g = torch.Generator(device=dev)
        g.manual_seed(synth.BASE_SEED + 4)
        rn = lambda shape, dt=torch.bfloat16: torch.randn(shape, device=dev, dtype=torch.float32, generator=g).to(dt)
        Q, K, V = (rn((wl.B, wl.Hq, wl.n, wl.d)) for _ in range(3))
        ga, gl = rn((wl.B, wl.Hq, wl.n), torch.float32), rn((wl.B, wl.Hq, wl.n), torch.float32)
        perm = torch.from_numpy(synth.permutations(1, 1, wl.n)).to(dev)
        dsa = sa.make_desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, sa.SA_WIN_SYM_CIRCULAR, 1, sa.SA_BF16, 0.0, 1, 1)
        dswa = sa.make_desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, sa.SA_WIN_ONE_SIDED, 1, sa.SA_BF16, 0.0, 1, 1)
        Y, Ysa, Yswa = (torch.empty_like(Q) for _ in range(3))
        Lsa = torch.empty((wl.B, wl.Hq, wl.n), device=dev, dtype=torch.float32)
        Lswa = torch.empty_like(Lsa)
        wsf = torch.empty(sa.sa_workspace_bytes(dsa, sa.SA_OP_GATED_FWD), device=dev, dtype=torch.uint8)
        call = lambda: sa.gated_sa_swa_fwd(dsa, dswa, Q, K, V, perm, ga, gl, Y, Ysa, Yswa, Lsa, Lswa, wsf)
    elif args.profile_op in ("gate_proj_fwd", "gate_proj_bwd"):
        # the gate projections of Eq. 6 + Eq. 5 at d_model = H * d = 1024 over the pre-training shape's tokens
        wl = synth.WORKLOADS["pretrain_fwdbwd_8k"]
        g = torch.Generator(device=dev)
        g.manual_seed(synth.BASE_SEED + 5)
        rn = lambda shape, sc=1.0: (torch.randn(shape, device=dev, dtype=torch.float32, generator=g) * sc).to(torch.bfloat16)
        dm = wl.Hq * wl.d
        Ysa, Yswa, dY = (rn((wl.B, wl.Hq, wl.n, wl.d)) for _ in range(3))
        Wsa, Wswa = rn((dm, dm), dm ** -0.5), rn((dm, dm), dm ** -0.5)
        Y, Gsa, Gswa, dYsa, dYswa = (torch.empty_like(Ysa) for _ in range(5))
        dWsa, dWswa = torch.empty_like(Wsa), torch.empty_like(Wswa)
        dsa = sa.make_desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, sa.SA_WIN_SYM_CIRCULAR, 1, sa.SA_BF16, 0.0, 1, 1)
        wsg = torch.empty(sa.sa_workspace_bytes(dsa, sa.SA_OP_GATE_PROJ_BWD), device=dev, dtype=torch.uint8)
        sa.sa_gate_proj_fwd(dsa, Ysa, Yswa, Wsa, Wswa, Y, Gsa, Gswa)
        if args.profile_op == "gate_proj_fwd":
            call = lambda: sa.sa_gate_proj_fwd(dsa, Ysa, Yswa, Wsa, Wswa, Y, Gsa, Gswa)
        else:
            call = lambda: sa.sa_gate_proj_bwd(dsa, Ysa, Yswa, Wsa, Wswa, Gsa, Gswa, dY, dYsa, dYswa, dWsa, dWswa, wsg)
    else:
        wl, call, keep = backward_setup(sa, synth, dev, "pretrain_fwdbwd_8k" if args.profile_op == "sa_bwd"
                                        else "qwen3_8b_prefill_32k")

    def step():
        if copy_src is not None:
            copy_dst.copy_(copy_src)
        call()
    _, mean_ms = time_op(step, args.steps, args.warmup)
    return {"op": args.profile_op, "workload": wl.name, "steps": args.steps, "warmup": args.warmup,
            "avg_step_ms": mean_ms, "calibrate_copy": bool(args.calibrate_copy)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--cpu-rows-per-head", type=int, default=32768)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-step", action="store_true", help="time the step only (for profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy before and between steps (a known-size kernel "
                         "for scaling the FETCH_SIZE / WRITE_SIZE counters; it also empties the caches)")
    ap.add_argument("--profile-op", choices=["sa_fwd", "sa_bwd", "sa_bwd_headline", "gated_fwd", "gate_proj_fwd", "gate_proj_bwd"],
                    default=None,
                    help="profiling runs: call this entry point --steps times (after --warmup) and print a short JSON "
                         "line; sa_fwd = the headline step, sa_bwd / gated_fwd = the pre-training shape B4 H16 n8192 "
                         "d64 w256, sa_bwd_headline = the backward at the headline shape, gate_proj_fwd / gate_proj_bwd = the gate "
                         "projections at d_model 1024 over the same tokens; honours --calibrate-copy")
    ap.add_argument("--table3", action="store_true",
                    help="instead of the headline step, run the sequence-length sweep of Sec. 4.3 / Table 3 "
                         "(SA, SWA, gated, full attention; forward + backward) and print it as one JSON line")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)

    from paper_2604_00754_amd import binding as sa
    from paper_2604_00754_amd import synth

    dev = "cuda:0"
    if args.table3:
        print(json.dumps(table3_sweep(sa, synth, dev)))
        return
    if args.profile_op in ("sa_bwd", "sa_bwd_headline", "gated_fwd", "gate_proj_fwd", "gate_proj_bwd"):
        print(json.dumps(profile_side_op(sa, synth, dev, args)))
        return
    wl = synth.WORKLOADS["qwen3_8b_prefill_32k"]
    g = torch.Generator(device=dev)
    g.manual_seed(synth.BASE_SEED)
    Q = torch.randn((wl.B, wl.Hq, wl.n, wl.d), device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16)
    K = torch.randn((wl.B, wl.Hkv, wl.n, wl.d), device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16)
    V = torch.randn((wl.B, wl.Hkv, wl.n, wl.d), device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16)
    perm = torch.from_numpy(synth.permutations(1, 1, wl.n)).to(dev)
    Y = torch.empty_like(Q)
    LSE = torch.empty((wl.B, wl.Hq, wl.n), device=dev, dtype=torch.float32)
    desc = sa.make_desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, sa.SA_WIN_SYM_CIRCULAR, 1, sa.SA_BF16,
                        0.0, 1, 1)

    copy_src = copy_dst = None
    if args.calibrate_copy:
        copy_src = torch.zeros(256 * 1024 * 1024, device=dev, dtype=torch.float32)  # 1 GiB
        copy_dst = torch.empty_like(copy_src)

    def step():
        if copy_src is not None:
            copy_dst.copy_(copy_src)
        sa.sa_fwd(desc, Q, K, V, perm, Y, LSE)

    # The side measurements run BEFORE the timed step: they are the same work as before in another order, and they
    # leave the GPU at its working clocks when the W warm-up steps and the K timed steps begin (after the few
    # milliseconds of a cold start the first launches of a short run are 10 - 15 % slower than the rest).
    W = band_slots(wl.n, wl.w, 0)
    band_flop = 4.0 * wl.n * W * wl.d * wl.B * wl.Hq            # QK^T and PV over the window band
    e = 2
    alg_bytes = wl.B * wl.n * (wl.Hq * 2 * wl.d * e + wl.Hkv * 2 * wl.d * e + wl.Hq * 4) + wl.n * 4
    bwd_block = None
    other = {}
    if not args.only_step:
        # clocks ramp over the first tens of milliseconds of load: bring them up before the first side measurement
        for _ in range(100):
            sa.sa_fwd(desc, Q, K, V, perm, Y, LSE)
        torch.cuda.synchronize()
        # the same call with the identity permutation and the one-sided causal window (plain SWA)
        swa_desc = sa.make_desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.w, sa.SA_WIN_ONE_SIDED, 1, sa.SA_BF16,
                                0.0, 1, 1)
        Y2 = torch.empty_like(Q)
        _, swa_ms = time_side(lambda: sa.swa_fwd(swa_desc, Q, K, V, Y2, None), max(10, args.steps // 4), 5)
        other = {"swa_fwd_ms": swa_ms, "swa_fwd_tokens_per_s": wl.B * wl.n / (swa_ms * 1e-3)}
        # gather + scatter with (almost) no attention work: w = 1, every token sees itself only
        w1_desc = sa.make_desc(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, 1, sa.SA_WIN_SYM_CIRCULAR, 1, sa.SA_BF16,
                               0.0, 1, 1)
        _, w1_ms = time_side(lambda: sa.sa_fwd(w1_desc, Q, K, V, perm, Y2, None), max(10, args.steps // 4), 5)
        other.update({"gather_scatter_w1_ms": w1_ms,
                      "gather_scatter_w1_GBps": alg_bytes / (w1_ms * 1e-3) / 1e9,
                      "gather_scatter_w1_frac_hbm": alg_bytes / (w1_ms * 1e-3) / 1e9 / PEAK_HBM_GBS})
        # the ceiling for that: gather + scatter alone (sa_permuted_copy), same rows, same index tensor
        _, pc_ms = time_side(lambda: sa.sa_permuted_copy(desc, Q, K, V, perm, Y2), max(10, args.steps // 4), 5)
        pc_bytes = alg_bytes - wl.B * wl.Hq * wl.n * 4  # no LSE
        other.update({"permuted_copy_ms": pc_ms, "permuted_copy_GBps": pc_bytes / (pc_ms * 1e-3) / 1e9,
                      "permuted_copy_frac_hbm": pc_bytes / (pc_ms * 1e-3) / 1e9 / PEAK_HBM_GBS})
        # a plain device-to-device copy of the same number of bytes (torch's copy kernel): what a read+write
        # stream with no index tensor reaches on this GPU
        flat_src = torch.empty(pc_bytes // 2, device=dev, dtype=torch.uint8)
        flat_dst = torch.empty_like(flat_src)
        _, cp_ms = time_side(lambda: flat_dst.copy_(flat_src), max(10, args.steps // 4), 5)
        other.update({"plain_copy_ms": cp_ms, "plain_copy_GBps": pc_bytes / (cp_ms * 1e-3) / 1e9})
        del flat_src, flat_dst
        # the headline launch with cold caches: a 1 GiB device copy between launches evicts L2 and MALL
        if copy_src is None:
            cs = torch.zeros(256 * 1024 * 1024, device=dev, dtype=torch.float32)
            cd = torch.empty_like(cs)
            cold = []
            for _ in range(10):
                cd.copy_(cs)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                sa.sa_fwd(desc, Q, K, V, perm, Y, LSE)
                b.record()
                torch.cuda.synchronize()
                cold.append(a.elapsed_time(b))
            other["cold_cache_ms"] = float(np.median(cold))
            del cs, cd
        # on-device permutation sampling (one layer, one permutation shared by the heads)
        sampled = torch.empty((1, 1, wl.n), device=dev, dtype=torch.int32)
        _, sp_ms = time_side(lambda: sa.sa_sample_perm(desc, 1, 0, sampled), 10, 2)
        d8k = sa.make_desc(4, 16, 16, 8192, 64, 256)
        sampled8k = torch.empty((1, 1, 8192), device=dev, dtype=torch.int32)
        _, sp8_ms = time_side(lambda: sa.sa_sample_perm(d8k, 1, 0, sampled8k), 10, 2)
        other.update({"sample_perm_n32768_ms": sp_ms, "sample_perm_n8192_ms": sp8_ms})
        # the same permutations through the bucketed O(n) path (needs a workspace)
        wss = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_SAMPLE_PERM), device=dev, dtype=torch.uint8)
        _, spw_ms = time_side(lambda: sa.sa_sample_perm(desc, 1, 0, sampled, wss), 10, 2)
        wss8 = torch.empty(sa.sa_workspace_bytes(d8k, sa.SA_OP_SAMPLE_PERM), device=dev, dtype=torch.uint8)
        _, spw8_ms = time_side(lambda: sa.sa_sample_perm(d8k, 1, 0, sampled8k, wss8), 10, 2)
        other.update({"sample_perm_ws_n32768_ms": spw_ms, "sample_perm_ws_n8192_ms": spw8_ms})
        del wss, wss8
        # RoPE on original positions for Q and K of the headline shape (out of place; table built once)
        table = torch.empty((wl.n, wl.d // 2, 2), device=dev, dtype=torch.float32)
        sa.sa_rope_table(wl.n, wl.d, 1e6, 0, table)
        Kr = torch.empty_like(K)
        _, rp_ms = time_side(lambda: sa.sa_rope(desc, Q, K, table, Y2, Kr), max(10, args.steps // 4), 5)
        rp_bytes = 2 * (Q.numel() + K.numel()) * 2
        other.update({"rope_qk_ms": rp_ms, "rope_qk_GBps": rp_bytes / (rp_ms * 1e-3) / 1e9,
                      "rope_qk_frac_hbm": rp_bytes / (rp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS})
        # the prefill sequence of Sec. 4.2 with the Q rotation fused: rotate K in memory, then sa_fwd_rope
        def rope_then_attention():
            sa.sa_rope(desc, None, K, table, None, Kr)
            sa.sa_fwd_rope(desc, Q, Kr, V, perm, table, Y, LSE)
        _, rf_ms = time_side(rope_then_attention, max(10, args.steps // 4), 5)
        other.update({"rope_k_plus_fwd_rope_ms": rf_ms, "rope_qk_ms_for_sum": rp_ms})
        # backward of the headline shape (not a workload of the paper, which trains at d = 64): dQ, dK, dV from dY
        dYh = torch.randn(Q.shape, device=dev, dtype=torch.float32).to(torch.bfloat16)
        dQh, dKh, dVh = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
        wsh = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_BWD), device=dev, dtype=torch.uint8)
        sa.sa_fwd(desc, Q, K, V, perm, Y, LSE)
        _, bw_ms = time_side(lambda: sa.sa_bwd(desc, None, Q, K, V, perm, None, None, Y, None, LSE, None, dYh,
                                             dQh, dKh, dVh, None, None, wsh), max(5, args.steps // 20), 2)
        other.update({"sa_bwd_headline_shape_ms": bw_ms})
        # the training sequence with RoPE on original positions, from unrotated Q and rotated K (what a forward with
        # the fused query rotation leaves): rotate Q in memory, sa_bwd, turn dQ and dK back in memory -- against
        # sa_bwd_rope (Q rotated while staged, dQ and dK turned back in the epilogues of the two kernels).  Timed
        # alternately; the forward that provides Y and LSE runs on the rotated rows.
        sa.sa_rope(desc, Q, K, table, Y2, Kr)
        sa.sa_fwd(desc, Y2, Kr, V, perm, Y, LSE)
        def rope_bwd_inverse_rope():
            sa.sa_rope(desc, Q, None, table, Y2, None)
            sa.sa_bwd(desc, None, Y2, Kr, V, perm, None, None, Y, None, LSE, None, dYh, dQh, dKh, dVh, None, None, wsh)
            sa.sa_rope(desc, dQh, dKh, table, dQh, dKh, inverse=1)
        wsr = torch.empty(sa.sa_workspace_bytes(desc, sa.SA_OP_BWD_ROPE), device=dev, dtype=torch.uint8)
        bu_ms, bf_ms = time_pair(rope_bwd_inverse_rope,
                                 lambda: sa.sa_bwd_rope(desc, Q, Kr, V, perm, table, Y, LSE, dYh, dQh, dKh, dVh, wsr,
                                                        dk_unrotated=1), max(5, args.steps // 20), 2)
        other.update({"rope_plus_sa_bwd_plus_inverse_rope_ms": bu_ms, "sa_bwd_rope_ms": bf_ms})
        del dYh, dQh, dKh, dVh, wsh, wsr, Y2, Kr, table
        # the decoding step that follows this prefill (Sec. 4.2): one new token per sequence over the whole
        # 32K-row cache of the same heads; and a batch of 16 sequences with 8K-row caches
        for name, Bd, nd in (("decode_32k", 1, wl.n), ("decode_b16_8k", 16, 8192)):
            dd = sa.make_desc(Bd, wl.Hq, wl.Hkv, nd, wl.d, 2)
            Kc = torch.randn((Bd, wl.Hkv, nd, wl.d), device=dev, dtype=torch.float32).to(torch.bfloat16)
            Vc = torch.randn((Bd, wl.Hkv, nd, wl.d), device=dev, dtype=torch.float32).to(torch.bfloat16)
            qd = torch.randn((Bd, wl.Hq, wl.d), device=dev, dtype=torch.float32).to(torch.bfloat16)
            Yd = torch.empty_like(qd)
            wsd = torch.empty(sa.sa_workspace_bytes(dd, sa.SA_OP_DECODE), device=dev, dtype=torch.uint8)
            _, dc_ms = time_side(lambda: sa.sa_decode_fwd(dd, qd, Kc, Vc, nd, Yd, None, wsd),
                                 max(10, args.steps // 4), 5)
            dc_bytes = 2 * Kc.numel() * 2 + 2 * qd.numel() * 2
            other.update({f"{name}_ms": dc_ms, f"{name}_GBps": dc_bytes / (dc_ms * 1e-3) / 1e9,
                          f"{name}_frac_hbm": dc_bytes / (dc_ms * 1e-3) / 1e9 / PEAK_HBM_GBS})
            del Kc, Vc, qd, Yd, wsd
        other.update(training_ops(sa, synth, dev, max(5, args.steps // 10)))
        other.update(long_prefill_ops(sa, synth, dev, max(3, args.steps // 40)))

    if not args.only_step:
        # the backward half of the metric, on the configuration the paper trains at
        bwd_block = backward_roofline(sa, synth, dev, max(10, args.steps), max(3, args.warmup))

    wall, launch_ms = time_op(step, args.steps, args.warmup)
    launch_samples = list(time_op.last_samples_ms)
    ms_per_step = wall * 1e3 / args.steps
    tokens_per_s = wl.B * wl.n / (wall / args.steps)
    assert torch.isfinite(Y.float()).all().item(), "sa_fwd produced non-finite values"

    tflops = band_flop / (launch_ms * 1e-3) / 1e12
    traffic, traffic_source = measured_traffic("sa_fwd", "qwen3_8b_prefill_32k")
    roofline = {"bound": "mfma", "kernel": "fwd_mfma_bf16_kernel<128, true, 2, false>", "achieved": tflops,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tflops / PEAK_BF16_TFLOPS,
                "traffic": traffic, "traffic_source": traffic_source,
                "algorithmic_flop": band_flop, "avg_launch_ms": launch_ms,
                "median_launch_ms": float(np.median(launch_samples)), "min_launch_ms": float(np.min(launch_samples)),
                "executed_flop": executed_flop(wl.n, wl.w, wl.d, wl.B, wl.Hq, BM=128 // heads_per_workgroup(wl),
                                               BN=32 if wl.d == 128 else 64),
                "caches": "not flushed between launches (see other_ops.cold_cache_ms)"}
    gbs = alg_bytes / (launch_ms * 1e-3) / 1e9
    roofline_hbm = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": gbs / PEAK_HBM_GBS, "algorithmic_bytes": alg_bytes}

    if not args.only_step:
        other["rope_qk_plus_fwd_ms"] = other.pop("rope_qk_ms_for_sum") + ms_per_step
        other["sa_fwdbwd_headline_shape_band_tflops"] = 3.5 * band_flop / ((ms_per_step + other["sa_bwd_headline_shape_ms"]) * 1e-3) / 1e12
    out = {"metric": METRIC, "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": "qwen3_8b_prefill_32k", "op": "sa_fwd", "B": wl.B, "Hq": wl.Hq,
                      "Hkv": wl.Hkv, "n": wl.n, "d": wl.d, "w": wl.w, "window": "sym_circular",
                      "causal_orig": 1, "perm": "one per layer, shared by heads"},
           "tflops_band": tflops, "pct_bf16_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS,
           "roofline": roofline, "roofline_hbm": roofline_hbm, "other_ops": other}
    if bwd_block is not None:
        out["roofline_bwd"] = bwd_block

    if not args.no_cpu_baseline and not args.only_step:
        base, rows, Yr = cpu_baseline(wl, Q, K, V, perm, args.cpu_rows_per_head)
        ri = torch.from_numpy(rows.astype(np.int64)).to(dev)
        got = Y[ri[:, 0], ri[:, 1], ri[:, 2]].float().cpu().numpy().astype(np.float64)
        diff = got - Yr
        base["gpu_vs_oracle_on_sample"] = {"max_abs": float(np.abs(diff).max()),
                                           "rel_l2": float(np.linalg.norm(diff) / np.linalg.norm(Yr))}
        out["cpu_baseline"] = base
        # the same launch priced by the pairs the mask leaves visible (counted by the oracle): about half the band
        out["tflops_visible_pairs"] = base["useful_flop"] / (launch_ms * 1e-3) / 1e12
    print(json.dumps(out))


if __name__ == "__main__":
    main()
