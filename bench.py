#!/usr/bin/env python3
"""Benchmark of the NTP shard hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input, at the
GPT-3-175B-shape configuration with the replica degraded from TP 8 to TP 7, rank 0:
  shard plans (host) -> MLP shard forward + backward (6 GEMMs, fused GeLU / GeLU')
  -> attention projection shard forward + backward (6 GEMMs)
  -> reshard of this rank's four weight gradients into the TP-8 layout.
`value` is the GEMM work of a step (logical 2*M*N*K flops) divided by the wall time of
the whole step, inputs resident in HBM.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E peak

# workload: GPT-3-175B-shape layer, full TP 8, degraded to TP 7, this GPU = rank 0
M, H, FFN, HEADS, HEAD_DIM, T_FULL, T_RED, RANK = 2048, 12288, 49152, 96, 128, 8, 7, 0


def build_state(torch, N):
    """Allocate and fill every buffer of the step (synthetic N(0,1) activations, N(0,0.02) weights)."""
    from paper_2504_06095_amd import inputs as I
    dev = "cuda"
    _, n_r = N.ntp_shard_plan(FFN, T_RED, RANK)
    ap = N.ntp_attn_shard_plan(HEADS, HEADS, HEAD_DIM, T_RED, RANK)
    wq, wo = ap["w_qkv"], ap["w_o"]
    # leading dimension of P, Y, dP: rows start on 128-byte lines (the library needs only a multiple of 8;
    # whole lines make the row-wise DMA of these matrices cheaper)
    ld = (n_r + 63) // 64 * 64

    def bf(name, shape, std):
        bits, _ = I.normal_bf16(0, "bench." + name, shape, std)
        return torch.from_numpy(bits.view("int16")).to(dev).view(torch.bfloat16)

    s = dict(n_r=n_r, wq=wq, wo=wo, ld=ld, ap=ap)
    s["X"], s["dZ"] = bf("X", (M, H), I.ACT_STD), bf("dZ", (M, H), I.ACT_STD)
    s["A_t"], s["B"] = bf("A_t", (n_r, H), I.WEIGHT_STD), bf("B", (n_r, H), I.WEIGHT_STD)
    s["Wqkv"], s["Wo"] = bf("Wqkv", (wq, H), I.WEIGHT_STD), bf("Wo", (wo, H), I.WEIGHT_STD)
    s["C"], s["dQKV"] = bf("C", (M, wo), I.ACT_STD), bf("dQKV", (M, wq), I.ACT_STD)
    e = lambda r, c, dt=torch.bfloat16: torch.empty(r, c, dtype=dt, device=dev)
    s["P"], s["Y"], s["dP"] = e(M, ld)[:, :n_r], e(M, ld)[:, :n_r], e(M, ld)[:, :n_r]
    s["Z"], s["dX"], s["Z2"], s["dX2"] = e(M, H), e(M, H), e(M, H), e(M, H)
    s["QKV"], s["dC"] = e(M, wq), e(M, wo)
    f32 = torch.float32
    s["dA_t"], s["dB"], s["dWqkv"], s["dWo"] = e(n_r, H, f32), e(n_r, H, f32), e(wq, H, f32), e(wo, H, f32)

    # reshard plan of this rank's gradients: TP 7 (only rank 0 present) -> TP 8 (ranks 0 and 1 receive)
    def reshard_job(src, rows, unit, kind, n_q=0, n_kv=0):
        spec = N.tensor_spec(rows, H, 0, unit, 4, kind, n_q, n_kv)
        srcs = [None] * T_RED
        srcs[RANK] = src
        dsts = [None] * T_FULL
        touched = {seg[1] for seg in N.ntp_reshard_segments(spec, T_RED, T_FULL) if seg[0] == RANK}
        for d in touched:
            if kind == N.binding.NTP_KIND_QKV_GQA:
                p = N.ntp_attn_shard_plan(n_q, n_kv, unit, T_FULL, d)
                w = p["w_qkv"]
            else:
                w = N.ntp_shard_plan(rows // unit, T_FULL, d)[1] * unit
            dsts[d] = e(w, H, f32)
        return spec, srcs, dsts

    K = N.binding
    s["reshard_jobs"] = [
        reshard_job(s["dA_t"], FFN, 1, K.NTP_KIND_PLAIN),
        reshard_job(s["dB"], FFN, 1, K.NTP_KIND_PLAIN),
        reshard_job(s["dWqkv"], 3 * HEADS * HEAD_DIM, HEAD_DIM, K.NTP_KIND_QKV_GQA, HEADS, HEADS),
        reshard_job(s["dWo"], HEADS * HEAD_DIM, HEAD_DIM, K.NTP_KIND_PLAIN),
    ]
    s["gemm_flops"] = 12.0 * M * H * n_r + 6.0 * M * H * (wq + wo)
    s["mlp_flops"] = 12.0 * M * H * n_r
    s["reshard_bytes"] = 2.0 * 4.0 * H * (2 * n_r + wq + wo)
    return s


def step(N, s):
    # a0: plans (host, pure)
    N.ntp_shard_plan(FFN, T_RED, RANK)
    N.ntp_attn_shard_plan(HEADS, HEADS, HEAD_DIM, T_RED, RANK)
    n_r, wq, wo = s["n_r"], s["wq"], s["wo"]
    # a1-a6: MLP shard
    N.ntp_mlp_shard_fwd(s["X"], s["A_t"], s["B"], s["P"], s["Y"], s["Z"], n_r)
    N.ntp_mlp_shard_bwd(s["dZ"], s["X"], s["A_t"], s["B"], s["P"], s["Y"], s["dP"], s["dX"], s["dA_t"], s["dB"], n_r)
    # a7-a9: attention projections
    N.ntp_attn_proj_shard_fwd(M, H, wq, wo, s["X"], s["Wqkv"], s["QKV"], s["C"], s["Wo"], s["Z2"])
    N.ntp_attn_proj_shard_bwd(M, H, wq, wo, s["dZ"], s["dQKV"], s["X"], s["C"], s["Wqkv"], s["Wo"], s["dC"], s["dX2"],
                              s["dWqkv"], s["dWo"])
    # a10: reshard this rank's gradients TP 7 -> TP 8
    for spec, srcs, dsts in s["reshard_jobs"]:
        N.ntp_reshard_grad(spec, T_RED, T_FULL, srcs, dsts)


def fused_state(N, s):
    """Row segments of this rank's four gradients in the destination (TP 8) shards of the step."""
    K = N.binding
    specs = [(FFN, 1, K.NTP_KIND_PLAIN, 0, 0), (FFN, 1, K.NTP_KIND_PLAIN, 0, 0),
             (3 * HEADS * HEAD_DIM, HEAD_DIM, K.NTP_KIND_QKV_GQA, HEADS, HEADS), (HEADS * HEAD_DIM, HEAD_DIM, K.NTP_KIND_PLAIN, 0, 0)]
    segs = []
    for (rows, unit, kind, q, kv), (_, _, dsts) in zip(specs, s["reshard_jobs"]):
        segs.append(N.ntp_reshard_row_segments(N.tensor_spec(rows, H, 0, unit, 4, kind, q, kv), T_RED, RANK, T_FULL, dsts))
    return segs


def step_fused(N, s, segs):
    """The same step with the gradient GEMMs storing straight into the TP-8 layout (no separate reshard pass)."""
    N.ntp_shard_plan(FFN, T_RED, RANK)
    N.ntp_attn_shard_plan(HEADS, HEADS, HEAD_DIM, T_RED, RANK)
    n_r, wq, wo = s["n_r"], s["wq"], s["wo"]
    N.ntp_mlp_shard_fwd(s["X"], s["A_t"], s["B"], s["P"], s["Y"], s["Z"], n_r)
    N.ntp_mlp_shard_bwd_resharded(s["dZ"], s["X"], s["A_t"], s["B"], s["P"], s["Y"], s["dP"], s["dX"], segs[0], segs[1], n_r)
    N.ntp_attn_proj_shard_fwd(M, H, wq, wo, s["X"], s["Wqkv"], s["QKV"], s["C"], s["Wo"], s["Z2"])
    N.ntp_attn_proj_shard_bwd_resharded(M, H, wq, wo, s["dZ"], s["dQKV"], s["X"], s["C"], s["Wqkv"], s["Wo"], s["dC"],
                                        s["dX2"], segs[2], segs[3])


def timed(torch, fn, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def kernel_table(N, torch, fn, steps):
    """Per-kernel average duration over `steps` steps, from HIP events on the launch stream."""
    torch.cuda.synchronize()
    N.ntp_kernel_timing_enable(True)
    for _ in range(steps):
        fn()
    recs = N.ntp_kernel_timing_read(1 << 16)
    N.ntp_kernel_timing_enable(False)
    table = {}
    for r in recs:
        t = table.setdefault(r["name"], dict(launches=0, ms=0.0, flops=0.0, bytes=0.0))
        t["launches"] += 1
        t["ms"] += r["ms"]
        t["flops"] += r["flops"]
        t["bytes"] += r["bytes"]
    return table


def cpu_baseline(s):
    """The oracle's GEMM work of the step on the host cores, same inputs, all tokens: MLP shard and
    attention projection shard, forward + backward, in float64.  (The reshard moves bits and is left out.)"""
    import numpy as np
    from oracle import ntp_oracle as O
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    X, dZ, A_i, B_i = f64(s["X"]), f64(s["dZ"]), f64(s["A_t"]).T.copy(), f64(s["B"])
    Wqkv_i, Wo_i, C, dQKV = f64(s["Wqkv"]).T.copy(), f64(s["Wo"]), f64(s["C"]), f64(s["dQKV"])
    t0 = time.perf_counter()
    P, Y, Z = O.mlp_shard_fwd(X, A_i, B_i)
    dP, dX, dA, dB = O.mlp_shard_bwd(dZ, X, A_i, B_i)
    QKV, Z2 = O.attn_proj_shard_fwd(X, Wqkv_i, C, Wo_i)
    dC, dX2, dWqkv, dWo = O.attn_proj_shard_bwd(dZ, dQKV, X, C, Wqkv_i, Wo_i)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    err = {}
    for name, want, got in (("Z", Z, s["Z"]), ("dX", dX, s["dX"]), ("dA_t", dA.T, s["dA_t"]), ("dB", dB, s["dB"]),
                            ("Y", Y, s["Y"]), ("dP", dP, s["dP"]), ("QKV", QKV, s["QKV"]), ("Zattn", Z2, s["Z2"]),
                            ("dC", dC, s["dC"]), ("dXattn", dX2, s["dX2"]), ("dWqkv", dWqkv.T, s["dWqkv"]),
                            ("dWo", dWo, s["dWo"])):
        g = got.float().cpu().numpy().astype(np.float64)
        err[name] = float(np.abs(g - want).max() / np.abs(want).max())
    return dict(value=s["gemm_flops"] / dt / 1e12, unit="TFLOP/s", cores=int(cores), kind="oracle",
                sample=f"all GEMM work of one step (MLP shard + attention projection shard, fwd+bwd, all {M} tokens, "
                       f"float64, {dt:.1f} s of host time: the whole workload, no sampling needed); reshard not included",
                seconds=dt), err


def reshard_stress(torch, N):
    """Config 5: all ranks of one 405B-shape layer's fp32 weight gradients, TP 71 -> 72 and back.
    fc1 and QKV gradients in the paper's orientation [H x width] (column blocks, odd widths),
    fc2 and out-proj gradients as row blocks."""
    Hh, F, nq, nkv, d, a, b = 16384, 53248, 128, 8, 128, 71, 72
    K = N.binding
    tensors = [  # rows, cols, partition_dim, unit, kind, n_q, n_kv
        (Hh, F, 1, 1, K.NTP_KIND_PLAIN, 0, 0),                      # fc1 dA
        (F, Hh, 0, 1, K.NTP_KIND_PLAIN, 0, 0),                      # fc2 dB
        (Hh, (nq + 2 * nkv) * d, 1, d, K.NTP_KIND_QKV_GQA, nq, nkv),  # QKV dW
        (nq * d, Hh, 0, d, K.NTP_KIND_PLAIN, 0, 0),                 # out-proj dW
    ]
    jobs = []
    total = {(a, b): 0.0, (b, a): 0.0}
    for rows, cols, pd, unit, kind, q, kv in tensors:
        spec = N.tensor_spec(rows, cols, pd, unit, 4, kind, q, kv)

        def width(tp, r):
            if kind == K.NTP_KIND_QKV_GQA:
                return N.ntp_attn_shard_plan(q, kv, unit, tp, r)["w_qkv"]
            return N.ntp_shard_plan((cols if pd else rows) // unit, tp, r)[1] * unit

        def shards(tp):
            return [torch.empty((rows, width(tp, r)) if pd else (width(tp, r), cols), dtype=torch.float32,
                                device="cuda").normal_(0, 1e-3) for r in range(tp)]
        sa, sb = shards(a), shards(b)
        jobs.append((spec, sa, sb))
        total[(a, b)] += 2.0 * 4 * sum(t.numel() for t in sb)
        total[(b, a)] += 2.0 * 4 * sum(t.numel() for t in sa)

    def run(fwd):
        for spec, sa, sb in jobs:
            if fwd:
                N.ntp_reshard_grad(spec, a, b, sa, sb)
            else:
                N.ntp_reshard_grad(spec, b, a, sb, sa)
    out = {}
    for key, fwd in (((a, b), True), ((b, a), False)):
        for _ in range(2):
            run(fwd)
        ms = timed(torch, lambda: run(fwd), 5)
        out[f"tp{key[0]}_to_tp{key[1]}"] = dict(ms=ms, GBps=total[key] / ms / 1e6, bytes=total[key])
    return out


def mapped_reshard_stress(torch, N):
    """The same 405B-shape fc1 / fc2 / out-proj gradients between the layouts of the comp / sync rank
    assignment (Sec. 3.1, Alg. 1) for a healthy TP-72 replica that synchronises with TP-71 replicas:
    compute layout (72 ranks, non-contiguous) -> sync layout (71 contiguous shards) and back.  Plans are
    built once, outside the timed region."""
    Hh, F, nq, d, t, tr = 16384, 53248, 128, 128, 72, 71
    tensors = [(Hh, F, 1, 1), (F, Hh, 0, 1), (nq * d, Hh, 0, d)]  # rows, cols, partition_dim, unit
    jobs = []
    total = 0.0
    for rows, cols, pd, unit in tensors:
        k = (cols if pd else rows) // unit
        comp, sync = N.ntp_comp_sync_plan(k, t, tr)
        spec = N.tensor_spec(rows, cols, pd, unit, 4)

        def shards(rank_of_unit, tp):
            cnt = [0] * tp
            for r in rank_of_unit:
                cnt[r] += 1
            return [torch.empty((rows, c * unit) if pd else (c * unit, cols), dtype=torch.float32,
                                device="cuda").normal_(0, 1e-3) for c in cnt]
        sc, ss = shards(comp, t), shards(sync, tr)
        plans = (N.ntp_reshard_plan_create(spec, t, comp, tr, sync), N.ntp_reshard_plan_create(spec, tr, sync, t, comp))
        for pl in plans:
            pl.ntp_reshard_plan_prepare()  # uploads the run table: the only allocation, outside the timed region
        jobs.append((*plans, sc, ss))
        total += 2.0 * 4 * rows * cols
    out = {}
    for key, fwd in (("comp_to_sync", True), ("sync_to_comp", False)):
        def run():
            for p_cs, p_sc, sc, ss in jobs:
                if fwd:
                    p_cs.ntp_reshard_plan_run(sc, ss)
                else:
                    p_sc.ntp_reshard_plan_run(ss, sc)
        for _ in range(2):
            run()
        ms = timed(torch, run, 5)
        out[key] = dict(ms=ms, GBps=total / ms / 1e6, bytes=total)
    for j in jobs:
        j[0].destroy()
        j[1].destroy()
    return out


def imbalance_sweep(torch, N, iters=8):
    """Second workload (`--imbalance-sweep`): every rank of a replica degraded from TP 8 to TP 7, 6 and 4
    at the prototype's layer shapes (hidden 6144 / 12288, head dimension 128, FFN 4 x hidden, 4K-16K tokens;
    Sec. 5.1 "Prototype evaluation").  Per (shape, t'): time of the slowest rank's layer shard (MLP +
    attention projections, forward + backward) over the mean over ranks, which is what the uneven split
    costs (Sec. 3.1: imbalance lowers the throughput of the reduced-TP replica), and over the TP-8 rank's
    time, which is what the lost GPUs cost.  A rank's time depends on its widths only, so each distinct
    (ffn columns, heads) pair is timed once."""
    dev = "cuda"
    out = []
    cache = {}

    def rank_ms(Mt, Hd, n_r, heads):
        key = (Mt, Hd, n_r, heads)
        if key in cache:
            return cache[key]
        bf = dict(dtype=torch.bfloat16, device=dev)
        wq, wo = 3 * heads * HEAD_DIM, heads * HEAD_DIM
        ld = (n_r + 7) // 8 * 8
        X, dZ = torch.randn(Mt, Hd, **bf), torch.randn(Mt, Hd, **bf)
        At, B = torch.randn(n_r, Hd, **bf) * 0.02, torch.randn(n_r, Hd, **bf) * 0.02
        Wqkv, Wo = torch.randn(wq, Hd, **bf) * 0.02, torch.randn(wo, Hd, **bf) * 0.02
        Cc, dQKV = torch.randn(Mt, wo, **bf), torch.randn(Mt, wq, **bf)
        e = lambda r, c, dt=torch.bfloat16: torch.empty(r, c, dtype=dt, device=dev)
        P, Y, dP = e(Mt, ld)[:, :n_r], e(Mt, ld)[:, :n_r], e(Mt, ld)[:, :n_r]
        Z, dX, Z2, dX2, QKV, dC = e(Mt, Hd), e(Mt, Hd), e(Mt, Hd), e(Mt, Hd), e(Mt, wq), e(Mt, wo)
        f32 = torch.float32
        dA, dB, dWq, dWo = e(n_r, Hd, f32), e(n_r, Hd, f32), e(wq, Hd, f32), e(wo, Hd, f32)

        def run():
            N.ntp_mlp_shard_fwd(X, At, B, P, Y, Z, n_r)
            N.ntp_mlp_shard_bwd(dZ, X, At, B, P, Y, dP, dX, dA, dB, n_r)
            N.ntp_attn_proj_shard_fwd(Mt, Hd, wq, wo, X, Wqkv, QKV, Cc, Wo, Z2)
            N.ntp_attn_proj_shard_bwd(Mt, Hd, wq, wo, dZ, dQKV, X, Cc, Wqkv, Wo, dC, dX2, dWq, dWo)
        for _ in range(3):
            run()
        cache[key] = timed(torch, run, iters)
        return cache[key]

    for Hd in (6144, 12288):
        heads, ffn = Hd // HEAD_DIM, 4 * Hd
        for Mt in (4096, 8192, 16384):
            base = rank_ms(Mt, Hd, ffn // T_FULL, heads // T_FULL)
            flops_layer = 12.0 * Mt * Hd * ffn + 6.0 * Mt * Hd * (4 * heads * HEAD_DIM)
            for tr in (7, 6, 4):
                per_rank = []
                for r in range(tr):
                    n_r = N.ntp_shard_plan(ffn, tr, r)[1]
                    q = N.ntp_attn_shard_plan(heads, heads, HEAD_DIM, tr, r)["q_cnt"]
                    per_rank.append(rank_ms(Mt, Hd, n_r, q))
                mx, mean = max(per_rank), sum(per_rank) / tr
                out.append(dict(hidden=Hd, tokens=Mt, full_tp=T_FULL, reduced_tp=tr, full_tp_rank_ms=base,
                                max_rank_ms=mx, mean_rank_ms=mean, max_over_mean=mx / mean,
                                slowdown_vs_full_tp=mx / base, ideal_slowdown=T_FULL / tr,
                                slowest_rank_TFLOPs=flops_layer / tr / mx / 1e9 if mx else None,
                                widths=sorted({(N.ntp_shard_plan(ffn, tr, r)[1],
                                                N.ntp_attn_shard_plan(heads, heads, HEAD_DIM, tr, r)["q_cnt"])
                                               for r in range(tr)})))
    return out


def attn_core_bench(torch, N):
    """Attention core (Eq. 5) of this rank's 14 local heads at the step's shape (one sequence of 2048 tokens),
    and at 8192 tokens where the quadratic part dominates; causal and unmasked, forward and backward."""
    out = {}
    for tokens in (M, 8192):
        for causal in (False, True):
            plan = N.ntp_attn_shard_plan(HEADS, HEADS, HEAD_DIM, T_RED, RANK)
            q = plan["q_cnt"]
            QKV = torch.randn(tokens, plan["w_qkv"], dtype=torch.bfloat16, device="cuda")
            Cc = torch.empty(tokens, plan["w_o"], dtype=torch.bfloat16, device="cuda")
            dC = torch.randn_like(Cc)
            dQKV = torch.empty_like(QKV)
            LSE = torch.empty(q, tokens, dtype=torch.float32, device="cuda")
            Delta = torch.empty_like(LSE)
            shp = N.attn_core_shape(1, tokens, plan, 1, causal)
            fwd = lambda: N.ntp_attn_core_shard_fwd(shp, QKV, Cc, LSE)
            bwd = lambda: N.ntp_attn_core_shard_bwd(shp, QKV, Cc, dC, LSE, Delta, dQKV)
            for _ in range(3):
                fwd()
                bwd()
            tf, tb = timed(torch, fwd, 10), timed(torch, bwd, 10)
            pair = (1.0 if causal else 2.0) * tokens * tokens * HEAD_DIM * q  # flops of one product over the visible pairs
            out[f"{tokens}_tokens_{'causal' if causal else 'full'}"] = dict(
                fwd_ms=tf, fwd_TFLOPs=2 * pair / tf / 1e9, bwd_ms=tb, bwd_TFLOPs=5 * pair / tb / 1e9,
                bwd_executed_TFLOPs=7 * pair / tb / 1e9)
    return out


def config_table(torch, N, iters=10):
    """`--config-table`: throughput of the shard calls at each of the five benchmark configurations (1: tiny MLP
    shard; 2: GPT-3-175B-shape MLP shard; 3: grouped-query attention shard at TP 30 of 32, projections and core;
    4: 405B-shape MLP shard at TP 71 of 72; 5 is the reshard stress of the default run)."""
    dev = "cuda"
    bf = dict(dtype=torch.bfloat16, device=dev)
    e = lambda r, c, dt=torch.bfloat16: torch.empty(r, c, dtype=dt, device=dev)
    rows = []

    def graphed(fwd, bwd):
        """ms of fwd + bwd replayed as one captured graph (what a launch-bound small layer gains from capture)."""
        side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            fwd(); bwd()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                fwd(); bwd()
        torch.cuda.synchronize()
        return timed(torch, graph.replay, iters)

    def mlp(tag, Mt, Hd, ffn, tp, rank):
        n_r = N.ntp_shard_plan(ffn, tp, rank)[1]
        ld = (n_r + 63) // 64 * 64
        X, dZ = torch.randn(Mt, Hd, **bf), torch.randn(Mt, Hd, **bf)
        At, B = torch.randn(n_r, Hd, **bf) * 0.02, torch.randn(n_r, Hd, **bf) * 0.02
        P, Y, dP = e(Mt, ld)[:, :n_r], e(Mt, ld)[:, :n_r], e(Mt, ld)[:, :n_r]
        Z, dX = e(Mt, Hd), e(Mt, Hd)
        dA, dB = e(n_r, Hd, torch.float32), e(n_r, Hd, torch.float32)
        fwd = lambda: N.ntp_mlp_shard_fwd(X, At, B, P, Y, Z, n_r)
        bwd = lambda: N.ntp_mlp_shard_bwd(dZ, X, At, B, P, Y, dP, dX, dA, dB, n_r)
        for _ in range(3):
            fwd(); bwd()
        tf, tb = timed(torch, fwd, iters), timed(torch, bwd, iters)
        fl = 4.0 * Mt * Hd * n_r
        rows.append(dict(config=tag, call="mlp shard", tokens=Mt, hidden=Hd, width=n_r, fwd_ms=tf, fwd_TFLOPs=fl / tf / 1e9,
                         bwd_ms=tb, bwd_TFLOPs=2 * fl / tb / 1e9, fwd_bwd_frac_of_peak=3 * fl / (tf + tb) / 1e9 / BF16_MFMA_PEAK_TFLOPS,
                         graph_fwd_bwd_ms=graphed(fwd, bwd)))

    def attn(tag, Mt, Hd, n_q, n_kv, d, tp, rank):
        plan = N.ntp_attn_shard_plan(n_q, n_kv, d, tp, rank)
        wq, wo, q = plan["w_qkv"], plan["w_o"], plan["q_cnt"]
        X, dZ = torch.randn(Mt, Hd, **bf), torch.randn(Mt, Hd, **bf)
        Wqkv, Wo = torch.randn(wq, Hd, **bf) * 0.02, torch.randn(wo, Hd, **bf) * 0.02
        QKV, Cc, Z, dC, dX, dQKV = e(Mt, wq), e(Mt, wo), e(Mt, Hd), e(Mt, wo), e(Mt, Hd), e(Mt, wq)
        dWq, dWo = e(wq, Hd, torch.float32), e(wo, Hd, torch.float32)
        LSE, Delta = e(q, Mt, torch.float32), e(q, Mt, torch.float32)
        shp = N.attn_core_shape(1, Mt, plan, n_q // n_kv, True)

        def fwd():
            N.ntp_attn_proj_shard_fwd(Mt, Hd, wq, wo, X, Wqkv, QKV, None, None, None)
            N.ntp_attn_core_shard_fwd(shp, QKV, Cc, LSE)
            N.ntp_attn_proj_shard_fwd(Mt, Hd, wq, wo, None, None, None, Cc, Wo, Z)

        def bwd():
            N.ntp_attn_proj_shard_bwd(Mt, Hd, wq, wo, dZ, None, None, Cc, None, Wo, dC, None, None, dWo)
            N.ntp_attn_core_shard_bwd(shp, QKV, Cc, dC, LSE, Delta, dQKV)
            N.ntp_attn_proj_shard_bwd(Mt, Hd, wq, wo, None, dQKV, X, None, Wqkv, None, None, dX, dWq, None)
        for _ in range(3):
            fwd(); bwd()
        tf, tb = timed(torch, fwd, iters), timed(torch, bwd, iters)
        proj = 2.0 * Mt * Hd * (wq + wo)
        core = 2.0 * Mt * Mt * d * q  # causal: half of 4 S^2 d per head
        rows.append(dict(config=tag, call="attention shard (projections + causal core)", tokens=Mt, hidden=Hd, heads=q, w_qkv=wq,
                         fwd_ms=tf, fwd_TFLOPs=(proj + core) / tf / 1e9, bwd_ms=tb, bwd_TFLOPs=(2 * proj + 2.5 * core) / tb / 1e9,
                         fwd_bwd_frac_of_peak=(3 * proj + 3.5 * core) / (tf + tb) / 1e9 / BF16_MFMA_PEAK_TFLOPS,
                         graph_fwd_bwd_ms=graphed(fwd, bwd)))

    mlp("c1", 512, 1024, 4096, 7, 0)
    mlp("c2", 2048, 12288, 49152, 7, 0)
    attn("c3 rank 0 (3 heads)", 4096, 8192, 64, 8, 128, 30, 0)
    attn("c3 rank 29 (2 heads)", 4096, 8192, 64, 8, 128, 30, 29)
    mlp("c4", 8192, 16384, 53248, 71, 0)
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-reshard-stress", action="store_true")
    ap.add_argument("--no-mapped-reshard", action="store_true")
    ap.add_argument("--no-fused-step", action="store_true")
    ap.add_argument("--no-attn-core", action="store_true")
    ap.add_argument("--config-table", action="store_true",
                    help="time the shard calls at each benchmark configuration instead and print a JSON line of its own")
    ap.add_argument("--imbalance-sweep", action="store_true",
                    help="run the second workload instead (all ranks of TP 8 degraded to 7, 6, 4 at the prototype's shapes) "
                         "and print its own JSON line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB dense copy (calibration_copy_kernel): the yardstick for profiler byte counters")
    ap.add_argument("--no-workspace", action="store_true",
                    help="do not register a split-K workspace (skinny shard GEMMs then run unsplit)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the shard hot path of a single rank); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2504_06095_amd as N
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if not args.no_workspace:
        # 1 GiB for the fp32 partial sums of split-K shard GEMMs, held for the whole run
        N.ntp_set_workspace(torch.empty(256 << 20, dtype=torch.float32, device="cuda"))
    if args.config_table:
        print(json.dumps({"metric": "shard fwd / bwd TFLOP/s per benchmark configuration", "unit": "TFLOP/s", "n_gpus": 1,
                          "dtype": "bf16", "data": "synthetic", "rows": config_table(torch, N)}))
        return
    if args.imbalance_sweep:
        rows = imbalance_sweep(torch, N)
        print(json.dumps({"metric": "layer shard time of the slowest rank over the mean over ranks (MLP + attention "
                                    "projections, fwd+bwd), all ranks of a TP-8 replica degraded to TP 7/6/4",
                          "unit": "ratio", "n_gpus": 1, "dtype": "bf16", "data": "synthetic", "higher_is_better": False,
                          "value": max(r["max_over_mean"] for r in rows), "rows": rows}))
        return
    s = build_state(torch, N)
    fn = lambda: step(N, s)
    for _ in range(args.warmup):
        fn()
    ms = timed(torch, fn, args.steps)
    value = s["gemm_flops"] / ms / 1e9

    # per-kernel durations over the same number of steps (HIP events on the launch stream)
    table = kernel_table(N, torch, fn, args.steps)
    gemms = {k: v for k, v in table.items() if k.startswith("gemm_")}
    dom_name = max(gemms, key=lambda k: gemms[k]["ms"])
    dom = gemms[dom_name]
    achieved = dom["flops"] / dom["ms"] / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(dom_name)
        except Exception:
            traffic = None
    roofline = dict(bound="mfma", kernel=dom_name, achieved=achieved, peak=BF16_MFMA_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=achieved / BF16_MFMA_PEAK_TFLOPS, traffic=traffic, launches_per_step=dom["launches"] / args.steps,
                    avg_launch_ms=dom["ms"] / dom["launches"], flops_per_launch=dom["flops"] / dom["launches"])
    gemm_ms = sum(v["ms"] for v in gemms.values()) / args.steps
    rs = [v for k, v in table.items() if k.startswith("reshard_")]
    parts = dict(gemm_ms_per_step=gemm_ms, gemm_TFLOPs=s["gemm_flops"] / gemm_ms / 1e9,
                 gemm_frac_of_peak=s["gemm_flops"] / gemm_ms / 1e9 / BF16_MFMA_PEAK_TFLOPS)
    if rs:
        rms = sum(v["ms"] for v in rs) / args.steps
        parts.update(reshard_ms_per_step=rms, reshard_GBps=sum(v["bytes"] for v in rs) / args.steps / rms / 1e6)
    kernels = {k: dict(avg_ms=v["ms"] / v["launches"], launches_per_step=v["launches"] / args.steps,
                       TFLOPs=(v["flops"] / v["ms"] / 1e9) if v["flops"] else None,
                       GBps=(v["bytes"] / v["ms"] / 1e6) if v["bytes"] else None) for k, v in table.items()}

    out = {
        "metric": "shard fwd+bwd TFLOP/s (% bf16 MFMA peak); reshard GB/s (% HBM peak)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "c2-gpt3-175b-shape layer shard, TP 8 degraded to TP 7, rank 0: MLP 2048x12288x7022 "
                               "fwd+bwd + attention projections (96 heads x 128, 14 on this rank) fwd+bwd + reshard "
                               "of the rank's dW (fp32) into the TP-8 layout",
                   "tokens": M, "hidden": H, "ffn": FFN, "n_r": s["n_r"], "w_qkv": s["wq"], "w_o": s["wo"],
                   "full_tp": T_FULL, "reduced_tp": T_RED, "rank": RANK,
                   "split_k_workspace_bytes": 0 if args.no_workspace else 1 << 30},
        "frac_of_bf16_peak": value / BF16_MFMA_PEAK_TFLOPS,
        "roofline": roofline, "parts": parts, "kernels": kernels,
    }
    if not args.no_fused_step:
        # destination shards as the unfused step leaves them (rows fed by other ranks keep a marker), then the
        # fused step must reproduce them bit for bit
        def mark():
            for _, _, dsts in s["reshard_jobs"]:
                for d in dsts:
                    if d is not None:
                        d.fill_(7.0)
        mark()
        fn()
        want = [[None if d is None else d.clone() for d in dsts] for _, _, dsts in s["reshard_jobs"]]
        mark()
        segs = fused_state(N, s)
        ffn = lambda: step_fused(N, s, segs)
        for _ in range(max(3, args.warmup // 4)):
            ffn()
        fms = timed(torch, ffn, args.steps)
        same = all(torch.equal(d.view(torch.int32), w.view(torch.int32)) for (_, _, dsts), ws in zip(s["reshard_jobs"], want) for d, w in zip(dsts, ws)
                   if d is not None)
        out["fused_reshard_step"] = dict(
            what="same step with the four gradient GEMMs storing straight into the TP-8 layout (no reshard pass)",
            ms_per_step=fms, value=s["gemm_flops"] / fms / 1e9, unit="TFLOP/s", speedup_vs_step=ms / fms,
            destination_shards_bit_identical=bool(same))
    if args.calibrate_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            N.ntp_calibration_copy(b, a)
        cms = timed(torch, lambda: N.ntp_calibration_copy(b, a), 5)
        out["calibration_copy"] = dict(bytes_read=a.numel() * 4, bytes_written=a.numel() * 4, ms=cms,
                                       GBps=2.0 * a.numel() * 4 / cms / 1e6)
        del a, b
    if not args.no_reshard_stress:
        st = reshard_stress(torch, N)
        worst = min(st.values(), key=lambda v: v["GBps"])
        out["reshard_roofline"] = dict(bound="hbm", workload="c5: 405B-shape layer dW fp32, all ranks, TP 71<->72",
                                       achieved=worst["GBps"], peak=HBM_PEAK_GBPS, unit="GB/s",
                                       frac=worst["GBps"] / HBM_PEAK_GBPS, traffic=None, directions=st)
    if not args.no_mapped_reshard:
        st = mapped_reshard_stress(torch, N)
        worst = min(st.values(), key=lambda v: v["GBps"])
        out["mapped_reshard_roofline"] = dict(
            bound="hbm", workload="405B-shape fc1/fc2/out-proj dW fp32, all ranks, comp layout (TP 72) <-> sync layout (TP 71) "
                                  "of the comp/sync rank assignment",
            achieved=worst["GBps"], peak=HBM_PEAK_GBPS, unit="GB/s", frac=worst["GBps"] / HBM_PEAK_GBPS, traffic=None,
            directions=st)
    if not args.no_attn_core:
        ac = attn_core_bench(torch, N)
        best = max(v["fwd_TFLOPs"] for v in ac.values())
        out["attn_core_roofline"] = dict(
            bound="mfma", workload="attention core of the rank's 14 heads x 128, one sequence; algorithmic flops: 2 products "
                                   "forward, 5 backward over the visible (query, key) pairs (the backward executes 7)",
            achieved=best, peak=BF16_MFMA_PEAK_TFLOPS, unit="TFLOP/s", frac=best / BF16_MFMA_PEAK_TFLOPS, traffic=None,
            cases=ac)
    if not args.no_cpu_baseline:
        fn()  # make sure the device buffers hold this step's results
        torch.cuda.synchronize()
        cb, err = cpu_baseline(s)
        out["cpu_baseline"] = cb
        out["parity_max_rel_err_vs_oracle"] = err
    print(json.dumps(out))


if __name__ == "__main__":
    main()
