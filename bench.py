#!/usr/bin/env python3
"""Benchmark of the NTP shard hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input, at the
GPT-3-175B-shape configuration with the replica degraded from TP 8 to TP 7, rank 0:
  shard plans (host) -> MLP shard forward + backward (6 GEMMs, fused GeLU / GeLU')
  -> attention projection shard forward + backward (6 GEMMs)
  -> reshard of this rank's four weight gradients into the TP-8 layout.
`value` is the GEMM work of a step (logical 2*M*N*K flops) divided by the wall time of
the whole step, inputs resident in HBM.  The same JSON line carries, each timed with
events on the launch stream (5 warm-up + 20 timed calls, median and minimum):
  configs            every benchmark configuration's shard call, forward + backward
  c4_roofline        the dominant kernel of the 405B-shape MLP shard (TP 71 of 72)
  reshard_roofline   the 405B-shape layer's gradients, all ranks, TP 71 <-> 72
  imbalance          all ranks of a TP-8 replica degraded to TP 7 at a prototype shape
  attn_core_roofline the attention core at the step's own shape
Every input comes from the keyed Philox generator of paper_2504_06095_amd/inputs.py, seed 0.
`--sections a,b,...` restricts the run (for profiler passes over one part).  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import statistics
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E peak
SEED = 0
WARM, TIMED = 5, 20             # per-call timing: warm-up and timed iterations

# workload of the step: GPT-3-175B-shape layer, full TP 8, degraded to TP 7, this GPU = rank 0
M, H, FFN, HEADS, HEAD_DIM, T_FULL, T_RED, RANK = 2048, 12288, 49152, 96, 128, 8, 7, 0

ALL_SECTIONS = ("step", "fused", "configs", "imbalance", "reshard", "mapped", "attn", "ceiling", "cpu")


# ---- seeded inputs ------------------------------------------------------------------------
def dev_bf16(torch, name, shape, std):
    """bf16 device tensor of N(0, std^2) values from the keyed generator (seed 0, keyed by name)."""
    from paper_2504_06095_amd import inputs as I
    bits, _ = I.normal_bf16(SEED, "bench." + name, shape, std)
    return torch.from_numpy(bits.view("int16")).to("cuda").view(torch.bfloat16)


_f32_blocks = {}


def dev_f32_tiled(torch, name, shape, std, block=1 << 24):
    """fp32 device tensor filled by repeating one seeded block of 16 Mi values (for the multi-GB gradient
    tensors of the reshard sections, whose bits only have to be distinct and reproducible)."""
    from paper_2504_06095_amd import inputs as I
    if name not in _f32_blocks:
        _f32_blocks[name] = torch.from_numpy(I.normal_f32(SEED, "bench." + name, (block,), std)).to("cuda")
    src = _f32_blocks[name]
    out = torch.empty(shape, dtype=torch.float32, device="cuda")
    flat = out.view(-1)
    for s in range(0, flat.numel(), block):
        e = min(flat.numel(), s + block)
        flat[s:e].copy_(src[: e - s])
    return out


def empty(torch, r, c, dt=None):
    return torch.empty(r, c, dtype=dt or torch.bfloat16, device="cuda")


# ---- timing ---------------------------------------------------------------------------------
def wall_ms(torch, fn, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def event_ms(torch, fn, warm=WARM, timed=TIMED):
    """Per-call durations (ms) between two events on the launch stream; returns (median, min)."""
    for _ in range(warm):
        fn()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(timed)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = [a.elapsed_time(b) for a, b in evs]
    return statistics.median(ts), min(ts)


def kernel_table(N, torch, fn, steps):
    """Per-kernel average duration over `steps` calls of fn, from HIP events on the launch stream."""
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


def traffic_of(section, kernel_name):
    """HBM-side bytes per launch of a kernel in one section of this benchmark, from the committed profiler summary
    (profiles/traffic.json, written from two rocprofv3 --pmc passes per section; its `source` entry names them), or
    None when that pass did not see this kernel (e.g. after a change of the launcher's tile choice)."""
    try:
        t = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
        return t.get(section, {}).get(kernel_name)
    except Exception:
        return None


def mfma_roofline(table, steps, section):
    gemms = {k: v for k, v in table.items() if k.startswith("gemm_")}
    if not gemms:
        return None
    name = max(gemms, key=lambda k: gemms[k]["ms"])
    d = gemms[name]
    achieved = d["flops"] / d["ms"] / 1e9
    return dict(bound="mfma", kernel=name, achieved=achieved, peak=BF16_MFMA_PEAK_TFLOPS, unit="TFLOP/s",
                frac=achieved / BF16_MFMA_PEAK_TFLOPS, traffic=traffic_of(section, name), launches_per_step=d["launches"] / steps,
                avg_launch_ms=d["ms"] / d["launches"], flops_per_launch=d["flops"] / d["launches"])


class ClockSampler:
    """Samples the GPU's shader clock while the timed work runs, from the driver's sysfs file pp_dpm_sclk (the line
    marked with * is the clock the power management runs the shader engines at just then); reports None where
    the file is not readable."""

    def __init__(self):
        paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.path = paths[0] if paths else None
        self.samples, self._stop, self._thr = [], threading.Event(), None

    def _read(self):
        for line in open(self.path).read().splitlines():
            if "*" in line:
                return float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        return None

    def _run(self):
        while not self._stop.is_set():
            try:
                v = self._read()
                if v:
                    self.samples.append(v)
            except Exception:
                pass
            time.sleep(0.001)

    def __enter__(self):
        if self.path:
            self._thr = threading.Thread(target=self._run, daemon=True)
            self._thr.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        if self._thr:
            self._thr.join()

    def summary(self):
        if not self.samples:
            return None
        s = sorted(self.samples)
        return dict(median_mhz=s[len(s) // 2], min_mhz=s[0], max_mhz=s[-1], samples=len(s), source=self.path,
                    nominal_mhz=2400.0)


# ---- the step ---------------------------------------------------------------------------------
def build_state(torch, N):
    """Allocate and fill every buffer of the step (seeded N(0,1) activations, N(0,0.02) weights)."""
    from paper_2504_06095_amd import inputs as I
    _, n_r = N.ntp_shard_plan(FFN, T_RED, RANK)
    ap = N.ntp_attn_shard_plan(HEADS, HEADS, HEAD_DIM, T_RED, RANK)
    wq, wo = ap["w_qkv"], ap["w_o"]
    # leading dimension of P, Y, dP: rows start on 128-byte lines (the library needs only a multiple of 8;
    # whole lines make the row-wise DMA of these matrices cheaper)
    ld = (n_r + 63) // 64 * 64
    bf = lambda name, shape, std: dev_bf16(torch, name, shape, std)
    e = lambda r, c, dt=None: empty(torch, r, c, dt)
    s = dict(n_r=n_r, wq=wq, wo=wo, ld=ld, ap=ap)
    s["X"], s["dZ"] = bf("X", (M, H), I.ACT_STD), bf("dZ", (M, H), I.ACT_STD)
    s["A_t"], s["B"] = bf("A_t", (n_r, H), I.WEIGHT_STD), bf("B", (n_r, H), I.WEIGHT_STD)
    s["Wqkv"], s["Wo"] = bf("Wqkv", (wq, H), I.WEIGHT_STD), bf("Wo", (wo, H), I.WEIGHT_STD)
    s["C"], s["dQKV"] = bf("C", (M, wo), I.ACT_STD), bf("dQKV", (M, wq), I.ACT_STD)
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
                w = N.ntp_attn_shard_plan(n_q, n_kv, unit, T_FULL, d)["w_qkv"]
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
    avail = len(os.sched_getaffinity(0))  # host cores available to this process
    blas_threads = None
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        pass
    err = {}
    for name, want, got in (("Z", Z, s["Z"]), ("dX", dX, s["dX"]), ("dA_t", dA.T, s["dA_t"]), ("dB", dB, s["dB"]),
                            ("Y", Y, s["Y"]), ("dP", dP, s["dP"]), ("QKV", QKV, s["QKV"]), ("Zattn", Z2, s["Z2"]),
                            ("dC", dC, s["dC"]), ("dXattn", dX2, s["dX2"]), ("dWqkv", dWqkv.T, s["dWqkv"]),
                            ("dWo", dWo, s["dWo"])):
        g = got.float().cpu().numpy().astype(np.float64)
        err[name] = float(np.abs(g - want).max() / np.abs(want).max())
    # threads the oracle's matrix products actually ran on: the BLAS pool, which cannot exceed the cores available
    cores = min(avail, blas_threads) if blas_threads else avail
    return dict(value=s["gemm_flops"] / dt / 1e12, unit="TFLOP/s", cores=int(cores), cores_available=avail,
                blas_threads=blas_threads, kind="oracle",
                sample=f"all GEMM work of one step (MLP shard + attention projection shard, fwd+bwd, all {M} tokens, "
                       f"float64, {dt:.1f} s of host time: the whole workload, no sampling needed); reshard not included",
                seconds=dt), err


# ---- every benchmark configuration -----------------------------------------------------------
def _activation(torch, cache, name, Mt, Hd):
    """X / dZ of one (tokens, hidden) shape: shared by every shard that is timed at that shape."""
    from paper_2504_06095_amd import inputs as I
    key = (name, Mt, Hd)
    if key not in cache:
        cache[key] = dev_bf16(torch, f"{name}.{Mt}x{Hd}", (Mt, Hd), I.ACT_STD)
    return cache[key]


class MlpShard:
    """Buffers and calls of one MLP shard (seeded inputs)."""

    def __init__(self, torch, N, tag, Mt, Hd, n_r, cache, ld_pad=64):
        from paper_2504_06095_amd import inputs as I
        self.N, self.Mt, self.Hd, self.n_r = N, Mt, Hd, n_r
        ld = (n_r + ld_pad - 1) // ld_pad * ld_pad
        self.X, self.dZ = _activation(torch, cache, "X", Mt, Hd), _activation(torch, cache, "dZ", Mt, Hd)
        self.At = dev_bf16(torch, f"{tag}.A_t", (n_r, Hd), I.WEIGHT_STD)
        self.B = dev_bf16(torch, f"{tag}.B", (n_r, Hd), I.WEIGHT_STD)
        e = lambda r, c, dt=None: empty(torch, r, c, dt)
        self.P, self.Y, self.dP = e(Mt, ld)[:, :n_r], e(Mt, ld)[:, :n_r], e(Mt, ld)[:, :n_r]
        self.Z, self.dX = e(Mt, Hd), e(Mt, Hd)
        self.dA, self.dB = e(n_r, Hd, torch.float32), e(n_r, Hd, torch.float32)
        self.flops = 12.0 * Mt * Hd * n_r

    def fwd(self):
        self.N.ntp_mlp_shard_fwd(self.X, self.At, self.B, self.P, self.Y, self.Z, self.n_r)

    def bwd(self):
        self.N.ntp_mlp_shard_bwd(self.dZ, self.X, self.At, self.B, self.P, self.Y, self.dP, self.dX, self.dA, self.dB, self.n_r)

    def run(self):
        self.fwd()
        self.bwd()


class AttnShard:
    """Buffers and calls of one attention shard of q query heads and kv KV heads (w_qkv = (q + 2 kv) d): the
    projections and, when `core_shape` is given, the attention core between them."""

    def __init__(self, torch, N, tag, Mt, Hd, q, kv, d, cache, core_shape=None):
        from paper_2504_06095_amd import inputs as I
        self.N, self.Mt, self.Hd, self.shape = N, Mt, Hd, core_shape
        self.wq, self.wo, self.q = (q + 2 * kv) * d, q * d, q
        wq, wo = self.wq, self.wo
        self.X, self.dZ = _activation(torch, cache, "X", Mt, Hd), _activation(torch, cache, "dZ", Mt, Hd)
        self.Wqkv = dev_bf16(torch, f"{tag}.Wqkv", (wq, Hd), I.WEIGHT_STD)
        self.Wo = dev_bf16(torch, f"{tag}.Wo", (wo, Hd), I.WEIGHT_STD)
        e = lambda r, c, dt=None: empty(torch, r, c, dt)
        self.QKV, self.Z, self.dC, self.dX = e(Mt, wq), e(Mt, Hd), e(Mt, wo), e(Mt, Hd)
        if core_shape is None:  # the core's outputs are inputs of the projection calls then
            self.C = dev_bf16(torch, f"{tag}.C", (Mt, wo), I.ACT_STD)
            self.dQKV = dev_bf16(torch, f"{tag}.dQKV", (Mt, wq), I.ACT_STD)
        else:
            self.C, self.dQKV = e(Mt, wo), e(Mt, wq)
        self.dWq, self.dWo = e(wq, Hd, torch.float32), e(wo, Hd, torch.float32)
        self.LSE, self.Delta = e(q, Mt, torch.float32), e(q, Mt, torch.float32)
        proj = 2.0 * Mt * Hd * (wq + wo)
        core = 2.0 * Mt * Mt * d * q if core_shape is not None else 0.0  # causal: half of 4 S^2 d per head
        self.flops = 3 * proj + 3.5 * core

    def fwd(self):
        N, Mt, Hd, wq, wo = self.N, self.Mt, self.Hd, self.wq, self.wo
        if self.shape is None:
            N.ntp_attn_proj_shard_fwd(Mt, Hd, wq, wo, self.X, self.Wqkv, self.QKV, self.C, self.Wo, self.Z)
            return
        N.ntp_attn_proj_shard_fwd(Mt, Hd, wq, wo, self.X, self.Wqkv, self.QKV, None, None, None)
        N.ntp_attn_core_shard_fwd(self.shape, self.QKV, self.C, self.LSE)
        N.ntp_attn_proj_shard_fwd(Mt, Hd, wq, wo, None, None, None, self.C, self.Wo, self.Z)

    def bwd(self):
        N, Mt, Hd, wq, wo = self.N, self.Mt, self.Hd, self.wq, self.wo
        if self.shape is None:
            N.ntp_attn_proj_shard_bwd(Mt, Hd, wq, wo, self.dZ, self.dQKV, self.X, self.C, self.Wqkv, self.Wo, self.dC, self.dX,
                                      self.dWq, self.dWo)
            return
        N.ntp_attn_proj_shard_bwd(Mt, Hd, wq, wo, self.dZ, None, None, self.C, None, self.Wo, self.dC, None, None, self.dWo)
        N.ntp_attn_core_shard_bwd(self.shape, self.QKV, self.C, self.dC, self.LSE, self.Delta, self.dQKV)
        N.ntp_attn_proj_shard_bwd(Mt, Hd, wq, wo, None, self.dQKV, self.X, None, self.Wqkv, None, None, self.dX, self.dWq, None)

    def run(self):
        self.fwd()
        self.bwd()


def time_shard(torch, sh):
    med, mn = event_ms(torch, sh.run)
    fmed, _ = event_ms(torch, sh.fwd, 2, 10)
    bmed, _ = event_ms(torch, sh.bwd, 2, 10)
    return dict(fwd_bwd_ms=med, fwd_bwd_ms_min=mn, fwd_ms=fmed, bwd_ms=bmed, flops=sh.flops, TFLOPs=sh.flops / med / 1e9,
                frac_of_bf16_peak=sh.flops / med / 1e9 / BF16_MFMA_PEAK_TFLOPS)


def config_section(torch, N):
    """Shard call of every benchmark configuration, forward + backward: 1 tiny MLP shard; 2 GPT-3-175B-shape MLP
    shard; 3 grouped-query attention shard at TP 30 of 32 (projections and causal core) for the three kinds of
    rank, and the TP-32 rank; 4 405B-shape MLP shard at TP 71 and at TP 72.  Returns (table, roofline of config 4's
    dominant kernel)."""
    from paper_2504_06095_amd import inputs as I
    out, cache = {}, {}
    w = I.C1_MLP
    out["c1"] = dict(call=f"MLP shard {w.M}x{w.H}x586 (TP 7 of 8, rank 0)", **time_shard(torch, MlpShard(torch, N, "c1", w.M, w.H, 586, cache)))
    cache.clear()
    w = I.C2_MLP
    out["c2"] = dict(call=f"MLP shard {w.M}x{w.H}x7022 (TP 7 of 8, rank 0)", **time_shard(torch, MlpShard(torch, N, "c2", w.M, w.H, 7022, cache)))
    cache.clear()
    w = I.C3_ATTN
    for key, tp, rank in (("c3_rank0", 30, 0), ("c3_rank2", 30, 2), ("c3_rank29", 30, 29), ("c3_tp32", 32, 0)):
        plan = N.ntp_attn_shard_plan(w.n_q, w.n_kv, w.d, tp, rank)
        shape = N.attn_core_shape(1, w.M, plan, w.n_q // w.n_kv, True)
        sh = AttnShard(torch, N, key, w.M, w.H, plan["q_cnt"], plan["kv_cnt"], w.d, cache, core_shape=shape)
        out[key] = dict(call=f"attention shard {w.M}x{w.H}, {sh.q} query heads (w_qkv {sh.wq}), projections + causal core, "
                             f"TP {tp} rank {rank}", **time_shard(torch, sh))
        del sh
    cache.clear()
    w = I.C4_MLP
    roof = None
    for key, tp, n_r in (("c4_tp71", 71, 750), ("c4_tp72", 72, 740)):
        sh = MlpShard(torch, N, key, w.M, w.H, n_r, cache)
        out[key] = dict(call=f"MLP shard {w.M}x{w.H}x{n_r} (TP {tp} of 72, rank 0)", **time_shard(torch, sh))
        if key == "c4_tp71":
            table = kernel_table(N, torch, sh.run, TIMED)
            roof = mfma_roofline(table, TIMED, "configs")
            roof["workload"] = out[key]["call"]
            roof["kernels"] = {k: dict(avg_ms=v["ms"] / v["launches"], launches_per_call=v["launches"] / TIMED,
                                       TFLOPs=v["flops"] / v["ms"] / 1e9 if v["flops"] else None) for k, v in table.items()}
        del sh
    cache.clear()
    torch.cuda.empty_cache()
    return out, roof


def imbalance_rows(torch, N, Hd, Mt, reduced=(7,)):
    """Every rank of a TP-8 replica degraded to TP t' at one prototype layer shape (Sec. 5.1 "Prototype evaluation":
    hidden 6144 / 12288, head dimension 128, FFN 4 x hidden, 4K-16K tokens).  Layer shard = MLP + attention
    projections, forward + backward.  A rank's time depends on its widths only, so each distinct (FFN columns,
    heads) pair is timed once."""
    heads, ffn = Hd // HEAD_DIM, 4 * Hd
    times, cache = {}, {}

    def rank_ms(n_r, q):
        if (n_r, q) not in times:
            mlp = MlpShard(torch, N, f"imb.{Hd}.{n_r}", Mt, Hd, n_r, cache, ld_pad=8)
            att = AttnShard(torch, N, f"imb.{Hd}.q{q}", Mt, Hd, q, q, HEAD_DIM, cache)

            def run():
                mlp.run()
                att.run()
            times[(n_r, q)] = event_ms(torch, run, 3, 10)[0]
        return times[(n_r, q)]

    base = rank_ms(ffn // T_FULL, heads // T_FULL)
    rows = []
    flops_layer = 12.0 * Mt * Hd * ffn + 6.0 * Mt * Hd * (4 * heads * HEAD_DIM)
    for tr in reduced:
        per_rank, widths = [], []
        for r in range(tr):
            n_r = N.ntp_shard_plan(ffn, tr, r)[1]
            q = N.ntp_attn_shard_plan(heads, heads, HEAD_DIM, tr, r)["q_cnt"]
            widths.append((n_r, q))
            per_rank.append(rank_ms(n_r, q))
        mx, mean = max(per_rank), sum(per_rank) / tr
        rows.append(dict(hidden=Hd, tokens=Mt, full_tp=T_FULL, reduced_tp=tr, full_tp_rank_ms=base, max_rank_ms=mx,
                         mean_rank_ms=mean, max_over_mean=mx / mean, slowdown_vs_full_tp=mx / base, ideal_slowdown=T_FULL / tr,
                         slowest_rank_TFLOPs=flops_layer / tr / mx / 1e9, widths=sorted(set(widths))))
    cache.clear()
    torch.cuda.empty_cache()
    return rows


def imbalance_sweep(torch, N):
    """`--imbalance-sweep`: the second workload in full (hidden 6144 / 12288 x 4K / 8K / 16K tokens x TP 7, 6, 4)."""
    rows = []
    for Hd in (6144, 12288):
        for Mt in (4096, 8192, 16384):
            rows += imbalance_rows(torch, N, Hd, Mt, (7, 6, 4))
    return rows


# ---- reshard sections --------------------------------------------------------------------------
def reshard_stress(torch, N):
    """Config 5: all ranks of one 405B-shape layer's fp32 weight gradients, TP 71 -> 72 and back.
    fc1 and QKV gradients in the paper's orientation [H x width] (column blocks, odd widths),
    fc2 and out-proj gradients as row blocks."""
    from paper_2504_06095_amd import inputs as I
    Hh, F, nq, nkv, d, a, b = I.C5_H, I.C5_FFN, I.C5_NQ, I.C5_NKV, I.C5_D, I.C5_TRED, I.C5_T
    K = N.binding
    tensors = [  # name, rows, cols, partition_dim, unit, kind, n_q, n_kv
        ("fc1", Hh, F, 1, 1, K.NTP_KIND_PLAIN, 0, 0), ("fc2", F, Hh, 0, 1, K.NTP_KIND_PLAIN, 0, 0),
        ("qkv", Hh, (nq + 2 * nkv) * d, 1, d, K.NTP_KIND_QKV_GQA, nq, nkv), ("out", nq * d, Hh, 0, d, K.NTP_KIND_PLAIN, 0, 0),
    ]
    jobs = []
    total = {(a, b): 0.0, (b, a): 0.0}
    for name, rows, cols, pd, unit, kind, q, kv in tensors:
        spec = N.tensor_spec(rows, cols, pd, unit, 4, kind, q, kv)

        def width(tp, r):
            if kind == K.NTP_KIND_QKV_GQA:
                return N.ntp_attn_shard_plan(q, kv, unit, tp, r)["w_qkv"]
            return N.ntp_shard_plan((cols if pd else rows) // unit, tp, r)[1] * unit

        def shards(tp):
            return [dev_f32_tiled(torch, "c5." + name, (rows, width(tp, r)) if pd else (width(tp, r), cols), I.GRAD_STD)
                    for r in range(tp)]
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
        med, mn = event_ms(torch, lambda: run(fwd))
        out[f"tp{key[0]}_to_tp{key[1]}"] = dict(ms=med, ms_min=mn, GBps=total[key] / med / 1e6, bytes=total[key])
    table = kernel_table(N, torch, lambda: run(True), 3)
    kern = {k: dict(avg_ms=v["ms"] / v["launches"], launches_per_pass=v["launches"] / 3, GBps=v["bytes"] / v["ms"] / 1e6,
                    bytes_per_launch=v["bytes"] / v["launches"], traffic=traffic_of("reshard", k)) for k, v in table.items()}
    return out, kern


def mapped_reshard_stress(torch, N):
    """The same 405B-shape fc1 / fc2 / out-proj gradients between the layouts of the comp / sync rank
    assignment (Sec. 3.1, Alg. 1) for a healthy TP-72 replica that synchronises with TP-71 replicas:
    compute layout (72 ranks, non-contiguous) -> sync layout (71 contiguous shards) and back.  Plans are
    built and prepared once, outside the timed region."""
    from paper_2504_06095_amd import inputs as I
    Hh, F, nq, d, t, tr = I.C5_H, I.C5_FFN, I.C5_NQ, I.C5_D, I.C5_T, I.C5_TRED
    tensors = [("fc1", Hh, F, 1, 1), ("fc2", F, Hh, 0, 1), ("out", nq * d, Hh, 0, d)]  # name, rows, cols, partition_dim, unit
    jobs = []
    total = 0.0
    for name, rows, cols, pd, unit in tensors:
        k = (cols if pd else rows) // unit
        comp, sync = N.ntp_comp_sync_plan(k, t, tr)
        spec = N.tensor_spec(rows, cols, pd, unit, 4)

        def shards(rank_of_unit, tp):
            cnt = [0] * tp
            for r in rank_of_unit:
                cnt[r] += 1
            return [dev_f32_tiled(torch, "c5." + name, (rows, c * unit) if pd else (c * unit, cols), I.GRAD_STD) for c in cnt]
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
        med, mn = event_ms(torch, run)
        out[key] = dict(ms=med, ms_min=mn, GBps=total / med / 1e6, bytes=total)
    for j in jobs:
        j[0].destroy()
        j[1].destroy()
    return out


def attn_core_bench(torch, N):
    """Attention core (Eq. 5) of this rank's 14 local heads at the step's shape (one sequence of 2048 tokens),
    and at 8192 tokens where the quadratic part dominates; causal and unmasked, forward and backward."""
    out = {}
    for tokens in (M, 8192):
        plan = N.ntp_attn_shard_plan(HEADS, HEADS, HEAD_DIM, T_RED, RANK)
        q = plan["q_cnt"]
        QKV = dev_bf16(torch, f"core.QKV.{tokens}", (tokens, plan["w_qkv"]), 1.0)
        dC = dev_bf16(torch, f"core.dC.{tokens}", (tokens, plan["w_o"]), 1.0)
        Cc = empty(torch, tokens, plan["w_o"])
        dQKV = torch.empty_like(QKV)
        LSE = empty(torch, q, tokens, torch.float32)
        Delta = torch.empty_like(LSE)
        for causal in (False, True):
            shp = N.attn_core_shape(1, tokens, plan, 1, causal)
            fwd = lambda: N.ntp_attn_core_shard_fwd(shp, QKV, Cc, LSE)
            bwd = lambda: N.ntp_attn_core_shard_bwd(shp, QKV, Cc, dC, LSE, Delta, dQKV)
            fwd()
            tf, tb = event_ms(torch, fwd)[0], event_ms(torch, bwd)[0]
            pair = (1.0 if causal else 2.0) * tokens * tokens * HEAD_DIM * q  # flops of one product over the visible pairs
            out[f"{tokens}_tokens_{'causal' if causal else 'full'}"] = dict(
                fwd_ms=tf, fwd_TFLOPs=2 * pair / tf / 1e9, bwd_ms=tb, bwd_TFLOPs=5 * pair / tb / 1e9,
                bwd_executed_TFLOPs=7 * pair / tb / 1e9)
    return out


def ceiling_probes(torch, N):
    """What the device sustains on the matrix pipe and on LDS reads, alone and in the GEMM kernels' own mix, with
    no global memory traffic (ntp_probe_rates): the bound that the power-limited clock and the LDS put on any
    schedule of the GEMM inner loop."""
    K = N.binding
    scratch = torch.empty(1 << 20, dtype=torch.float32, device="cuda")
    names = (("mfma_only", K.NTP_PROBE_MFMA), ("lds_read_b128", K.NTP_PROBE_LDS_B128), ("lds_read_tr_b64", K.NTP_PROBE_LDS_TR_B64),
             ("mfma_plus_lds_b128", K.NTP_PROBE_MFMA_LDS_B128), ("mfma_plus_lds_tr_b64", K.NTP_PROBE_MFMA_LDS_TR_B64))
    out = {}
    for name, which in names:
        N.ntp_probe_rates(which, scratch)  # settle the clock on this loop
        r = N.ntp_probe_rates(which, scratch)
        out[name] = dict(TFLOPs=r["tflops"] or None, frac_of_bf16_peak=(r["tflops"] / BF16_MFMA_PEAK_TFLOPS) or None,
                         lds_read_GBps_per_cu=r["lds_gbps_per_cu"] or None, mfma_per_turn=r["mfma_per_turn"],
                         lds_reads_per_turn=r["reads_per_turn"], ms=r["ms"])
    # one wavefront per SIMD doing matrix instructions, one doing a softmax's vector arithmetic, and both together:
    # how much of the vector work hides behind the matrix pipe (the attention core's ceiling)
    t = {}
    for name, which in (("matrix", K.NTP_PROBE_MFMA_1WAVE), ("softmax", K.NTP_PROBE_SOFTMAX_1WAVE), ("both", K.NTP_PROBE_MFMA_AND_SOFTMAX)):
        N.ntp_probe_rates(which, scratch)
        t[name] = N.ntp_probe_rates(which, scratch)["ms"]
    out["matrix_and_softmax_on_one_simd"] = dict(
        matrix_alone_ms=t["matrix"], softmax_alone_ms=t["softmax"], both_ms=t["both"],
        softmax_share_hidden=(t["matrix"] + t["softmax"] - t["both"]) / t["softmax"],
        what="per turn 32 matrix instructions on one wavefront per SIMD and the vector arithmetic of 16 scores per lane on another")
    return out


def workspace_wish(N):
    """As much workspace as any shard call that this benchmark times can use (ntp_workspace_bytes)."""
    from paper_2504_06095_amd import inputs as I
    K = N.binding
    wish = [N.ntp_workspace_bytes(K.NTP_CALL_MLP_SHARD, K.MlpShape(w.M, w.H, n_r, 0))
            for w, n_r in ((I.C1_MLP, 586), (I.C2_MLP, 7022), (I.C4_MLP, 750), (I.C4_MLP, 740))]
    w3 = I.C3_ATTN
    for tp, rank in ((30, 0), (30, 2), (30, 29), (32, 0)):
        p = N.ntp_attn_shard_plan(w3.n_q, w3.n_kv, w3.d, tp, rank)
        wish.append(N.ntp_workspace_bytes(K.NTP_CALL_ATTN_PROJ_SHARD, K.AttnShape(w3.M, w3.H, p["w_qkv"], p["w_o"])))
        wish.append(N.ntp_workspace_bytes(K.NTP_CALL_ATTN_CORE_SHARD, N.attn_core_shape(1, w3.M, p, w3.n_q // w3.n_kv, True)))
    ap7 = N.ntp_attn_shard_plan(HEADS, HEADS, HEAD_DIM, T_RED, RANK)
    wish.append(N.ntp_workspace_bytes(K.NTP_CALL_ATTN_PROJ_SHARD, K.AttnShape(M, H, ap7["w_qkv"], ap7["w_o"])))
    wish.append(N.ntp_workspace_bytes(K.NTP_CALL_ATTN_CORE_SHARD, N.attn_core_shape(1, M, ap7, 1, True)))
    return max(256, (max(wish) + 255) // 256 * 256)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--sections", default=",".join(ALL_SECTIONS),
                    help="comma-separated subset of: " + ", ".join(ALL_SECTIONS) + " (profiler passes use one at a time)")
    ap.add_argument("--imbalance-sweep", action="store_true",
                    help="run the second workload in full instead (all ranks of TP 8 degraded to 7, 6, 4 at the prototype's "
                         "shapes) and print its own JSON line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB dense copy (calibration_copy_kernel): the yardstick for profiler byte counters")
    ap.add_argument("--gemm-schedule", type=int, default=None,
                    help="NTP_OPT_GEMM_SCHEDULE override for A/B runs (1: the ring kernel's default schedule everywhere, 2: ping-pong)")
    ap.add_argument("--diagnostic-zero-operands", action="store_true",
                    help="step section only: run the step on all-zero operands instead (same instructions and memory traffic, almost no "
                         "switching power in the matrix pipe): shows how far the board's power limit holds the GEMM kernels back. "
                         "The line is marked as a diagnostic, not a result")
    ap.add_argument("--no-workspace", action="store_true",
                    help="give the handle no split-K workspace (skinny shard GEMMs then run unsplit)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the shard hot path of a single rank); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)
    sections = set(x for x in args.sections.split(",") if x)
    unknown = sections - set(ALL_SECTIONS)
    if unknown:
        print(f"bench.py: unknown sections {sorted(unknown)}", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2504_06095_amd as N
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.gemm_schedule is not None:
        N.ntp_set_option(N.binding.NTP_OPT_GEMM_SCHEDULE, args.gemm_schedule)
    ws_bytes = 0
    if not args.no_workspace:
        ws_bytes = workspace_wish(N)
        N.ntp_set_workspace(torch.empty(ws_bytes // 4, dtype=torch.float32, device="cuda"))
    if args.imbalance_sweep:
        rows = imbalance_sweep(torch, N)
        print(json.dumps({"metric": "layer shard time of the slowest rank over the mean over ranks (MLP + attention "
                                    "projections, fwd+bwd), all ranks of a TP-8 replica degraded to TP 7/6/4",
                          "unit": "ratio", "n_gpus": 1, "dtype": "bf16", "data": "synthetic", "higher_is_better": False,
                          "value": max(r["max_over_mean"] for r in rows), "rows": rows}))
        return

    info = N.ntp_device_info()
    out = {
        "metric": "shard fwd+bwd TFLOP/s (% bf16 MFMA peak); reshard GB/s (% HBM peak)",
        "value": None, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "c2-gpt3-175b-shape layer shard, TP 8 degraded to TP 7, rank 0: MLP 2048x12288x7022 "
                               "fwd+bwd + attention projections (96 heads x 128, 14 on this rank) fwd+bwd + reshard "
                               "of the rank's dW (fp32) into the TP-8 layout",
                   "tokens": M, "hidden": H, "ffn": FFN, "full_tp": T_FULL, "reduced_tp": T_RED, "rank": RANK,
                   "split_k_workspace_bytes": ws_bytes, "compute_units": info["compute_units"], "seed": SEED,
                   "sections": sorted(sections)},
    }
    s = None
    fn = None
    if sections & {"step", "fused", "cpu"}:
        s = build_state(torch, N)
        fn = lambda: step(N, s)
        out["config"].update(n_r=s["n_r"], w_qkv=s["wq"], w_o=s["wo"])
    if "step" in sections:
        if args.diagnostic_zero_operands:
            for k in ("X", "dZ", "A_t", "B", "Wqkv", "Wo", "C", "dQKV"):
                s[k].zero_()
            out["data"] = "all-zero operands (power diagnostic: not a benchmark result)"
        for _ in range(args.warmup):
            fn()
        with ClockSampler() as clk:
            ms = wall_ms(torch, fn, args.steps)
        value = s["gemm_flops"] / ms / 1e9
        out.update(value=value, ms_per_step=ms, frac_of_bf16_peak=value / BF16_MFMA_PEAK_TFLOPS)
        out["sustained_clock"] = clk.summary()
        # per-kernel durations over the same number of steps (HIP events on the launch stream)
        table = kernel_table(N, torch, fn, args.steps)
        out["roofline"] = mfma_roofline(table, args.steps, "step")
        gemms = {k: v for k, v in table.items() if k.startswith("gemm_")}
        gemm_ms = sum(v["ms"] for v in gemms.values()) / args.steps
        rs = [v for k, v in table.items() if k.startswith("reshard_")]
        parts = dict(gemm_ms_per_step=gemm_ms, gemm_TFLOPs=s["gemm_flops"] / gemm_ms / 1e9,
                     gemm_frac_of_peak=s["gemm_flops"] / gemm_ms / 1e9 / BF16_MFMA_PEAK_TFLOPS)
        if rs:
            rms = sum(v["ms"] for v in rs) / args.steps
            parts.update(reshard_ms_per_step=rms, reshard_GBps=sum(v["bytes"] for v in rs) / args.steps / rms / 1e6)
        out["parts"] = parts
        out["kernels"] = {k: dict(avg_ms=v["ms"] / v["launches"], launches_per_step=v["launches"] / args.steps,
                                  TFLOPs=(v["flops"] / v["ms"] / 1e9) if v["flops"] else None,
                                  GBps=(v["bytes"] / v["ms"] / 1e6) if v["bytes"] else None,
                                  frac=(v["flops"] / v["ms"] / 1e9 / BF16_MFMA_PEAK_TFLOPS) if v["flops"]
                                  else (v["bytes"] / v["ms"] / 1e6 / HBM_PEAK_GBPS)) for k, v in table.items()}
    if "fused" in sections:
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
        fms = wall_ms(torch, ffn, args.steps)
        same = all(torch.equal(d.view(torch.int32), w.view(torch.int32)) for (_, _, dsts), ws in zip(s["reshard_jobs"], want)
                   for d, w in zip(dsts, ws) if d is not None)
        out["fused_reshard_step"] = dict(
            what="same step with the four gradient GEMMs storing straight into the TP-8 layout (no reshard pass)",
            ms_per_step=fms, value=s["gemm_flops"] / fms / 1e9, unit="TFLOP/s",
            speedup_vs_step=(out["ms_per_step"] / fms) if out["ms_per_step"] else None, destination_shards_bit_identical=bool(same))
        del want
    if "cpu" in sections:
        fn()  # make sure the device buffers hold this step's results
        torch.cuda.synchronize()
        cb, err = cpu_baseline(s)
        out["cpu_baseline"] = cb
        out["parity_max_rel_err_vs_oracle"] = err
    s = fn = None
    torch.cuda.empty_cache()
    if args.calibrate_copy:
        a = dev_f32_tiled(torch, "calibration", (1 << 28,), 1.0)
        b = torch.empty_like(a)
        cms = event_ms(torch, lambda: N.ntp_calibration_copy(b, a), 3, 5)[0]
        out["calibration_copy"] = dict(bytes_read=a.numel() * 4, bytes_written=a.numel() * 4, ms=cms,
                                       GBps=2.0 * a.numel() * 4 / cms / 1e6)
        del a, b
    if "configs" in sections:
        out["configs"], out["c4_roofline"] = config_section(torch, N)
    if "imbalance" in sections:
        rows = imbalance_rows(torch, N, 12288, 8192, (7,))
        out["imbalance"] = dict(what="all ranks of a TP-8 replica degraded to TP 7, layer shard (MLP + attention projections, "
                                     "fwd+bwd) at hidden 12288, 8192 tokens; the full sweep is `bench.py --imbalance-sweep`",
                                **rows[0])
    if "attn" in sections:
        ac = attn_core_bench(torch, N)
        own = ac[f"{M}_tokens_causal"]  # the step's own shape: one sequence of 2048 tokens, decoder mask
        worst = min(own["fwd_TFLOPs"], own["bwd_TFLOPs"])
        out["attn_core_roofline"] = dict(
            bound="mfma", workload="attention core of the rank's 14 heads x 128 at the step's shape (one sequence of 2048 tokens, "
                                   "causal): the slower of forward and backward; algorithmic flops: 2 products forward, 5 backward "
                                   "over the visible (query, key) pairs (the backward executes 7)",
            achieved=worst, peak=BF16_MFMA_PEAK_TFLOPS, unit="TFLOP/s", frac=worst / BF16_MFMA_PEAK_TFLOPS, traffic=None,
            cases=ac)
        torch.cuda.empty_cache()
    if "ceiling" in sections:
        out["device_ceiling"] = ceiling_probes(torch, N)
    if "reshard" in sections:
        st, kern = reshard_stress(torch, N)
        worst = min(st.values(), key=lambda v: v["GBps"])
        traffic = None
        if kern and all(v["traffic"] is not None for v in kern.values()):
            traffic = sum(v["traffic"] * v["launches_per_pass"] for v in kern.values())
        out["reshard_roofline"] = dict(bound="hbm", workload="c5: 405B-shape layer dW fp32, all ranks, TP 71<->72 (slower direction)",
                                       achieved=worst["GBps"], peak=HBM_PEAK_GBPS, unit="GB/s",
                                       frac=worst["GBps"] / HBM_PEAK_GBPS, traffic=traffic,
                                       traffic_note="HBM-side bytes of one 71->72 pass (all its launches), from profiles/traffic.json",
                                       directions=st, kernels_71_to_72=kern)
        _f32_blocks.clear()
        torch.cuda.empty_cache()
    if "mapped" in sections:
        st = mapped_reshard_stress(torch, N)
        worst = min(st.values(), key=lambda v: v["GBps"])
        out["mapped_reshard_roofline"] = dict(
            bound="hbm", workload="405B-shape fc1/fc2/out-proj dW fp32, all ranks, comp layout (TP 72) <-> sync layout (TP 71) "
                                  "of the comp/sync rank assignment",
            achieved=worst["GBps"], peak=HBM_PEAK_GBPS, unit="GB/s", frac=worst["GBps"] / HBM_PEAK_GBPS, traffic=None,
            directions=st)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
