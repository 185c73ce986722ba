"""Seeded synthetic inputs for the NTP shard hot path.

This module only *makes data*: normal deviates from a counter-based generator
(Philox, keyed by seed and a tensor name), rounding of those deviates to the
bf16 grid, and the shapes of the paper-like workloads.  It holds none of the
method's arithmetic (no shard plan, no GEMM, no GeLU, no reshard), so that the
HIP path and the CPU oracle can both be fed from it without sharing logic.

Workload shapes follow the evaluation set-up of the paper (hidden 6144/12288,
FFN = 4 x hidden, head dim 128; Sec. 5.1) and the larger LLM shapes named in
the benchmark configurations (GPT-3-175B, 405B-class).
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass

import numpy as np


def _key(seed: int, name: str) -> list[int]:
    # Philox takes a 2x64-bit key: the seed and a stable hash of the tensor name.
    return [int(seed) & 0xFFFFFFFFFFFFFFFF, zlib.crc32(name.encode()) & 0xFFFFFFFF]


def normal_f32(seed: int, name: str, shape, std: float = 1.0) -> np.ndarray:
    """N(0, std^2) float32 array; the same (seed, name, shape) always gives the same values."""
    gen = np.random.Generator(np.random.Philox(key=_key(seed, name)))
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.float32)
    chunk = 1 << 26
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        gen.standard_normal(e - s, dtype=np.float32, out=out[s:e])
    if std != 1.0:
        out *= np.float32(std)
    return out.reshape(shape)


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns.

    This is the storage format of the inputs, not a step of the method.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding_bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding_bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to float32 (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(seed: int, name: str, shape, std: float = 1.0):
    """N(0, std^2) rounded to bf16.  Returns (bits uint16, values float32), both of `shape`."""
    bits = round_to_bf16_bits(normal_f32(seed, name, shape, std))
    return bits, bf16_bits_to_f32(bits)


@dataclass(frozen=True)
class MlpWorkload:
    """One MLP block: M tokens, hidden H, FFN width n, full TP t, reduced TP t_red."""
    name: str
    M: int
    H: int
    n: int
    t: int
    t_red: int


@dataclass(frozen=True)
class AttnWorkload:
    """One attention block's projections: M tokens, hidden H, n_q query heads, n_kv KV heads of size d."""
    name: str
    M: int
    H: int
    n_q: int
    n_kv: int
    d: int
    t: int
    t_red: int


# The benchmark configurations (synthetic shapes; values N(0,1) activations / N(0,0.02) weights, bf16).
C1_MLP = MlpWorkload("c1-small-mlp", M=512, H=1024, n=4096, t=8, t_red=7)
C2_MLP = MlpWorkload("c2-gpt3-175b-mlp", M=2048, H=12288, n=49152, t=8, t_red=7)
C3_ATTN = AttnWorkload("c3-gqa-attn", M=4096, H=8192, n_q=64, n_kv=8, d=128, t=32, t_red=30)
C4_MLP = MlpWorkload("c4-405b-mlp", M=8192, H=16384, n=53248, t=72, t_red=71)
# Reshard stress: one 405B-shape layer's weight gradients, TP 71 <-> 72.
C5_H, C5_FFN, C5_NQ, C5_NKV, C5_D, C5_T, C5_TRED = 16384, 53248, 128, 8, 128, 72, 71

ACT_STD = 1.0
WEIGHT_STD = 0.02
GRAD_STD = 1.0e-3
