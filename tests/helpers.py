"""Shared by the test files: build seeded inputs, run the HIP path and the oracle side by side.

The HIP path and the oracle meet only here.  Layout conversion between the paper's
orientation (A [H x n], columns partitioned) and the library's storage (A_t [n_r x H])
is done here, on the host, with numpy.
"""
from __future__ import annotations

import numpy as np

from oracle import ntp_oracle as O
from paper_2504_06095_amd import inputs as I

TOL = 2e-2  # max|gpu - oracle| / max|oracle|, the bound the benchmark statement fixes for bf16 GEMMs


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    denom = float(np.abs(want).max())
    if denom == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got.astype(np.float64) - want).max() / denom)


def round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


def to_dev_bf16(bits: np.ndarray, ld: int | None = None):
    """uint16 bit patterns [r, c] -> device bf16 tensor view [r, c] with row stride ld (pad poisoned with NaN)."""
    import torch
    r, c = bits.shape
    ld = c if ld is None else ld
    buf = torch.full((r, ld), float("nan"), dtype=torch.bfloat16, device="cuda")
    buf[:, :c] = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return buf[:, :c]


def dev_bf16_to_f64(t) -> np.ndarray:
    import torch
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


class MlpCase:
    """Inputs of one MLP shard in both representations."""

    def __init__(self, M, H, n, tp, rank, seed=0, tag="mlp"):
        self.M, self.H, self.n, self.tp, self.rank = M, H, n, tp, rank
        self.off, self.n_r = O.shard_plan(n, tp, rank)
        n_r = self.n_r
        # only this rank's slice of the weights is generated (named by its logical offset)
        self.X_bits, X = I.normal_bf16(seed, f"{tag}.X", (M, H), I.ACT_STD)
        self.At_bits, At = I.normal_bf16(seed, f"{tag}.A_t.{tp}.{rank}", (n_r, H), I.WEIGHT_STD)
        self.B_bits, B = I.normal_bf16(seed, f"{tag}.B.{tp}.{rank}", (n_r, H), I.WEIGHT_STD)
        self.dZ_bits, dZ = I.normal_bf16(seed, f"{tag}.dZ", (M, H), I.ACT_STD)
        self.X, self.dZ = X.astype(np.float64), dZ.astype(np.float64)
        self.A_i = At.astype(np.float64).T.copy()  # paper orientation [H x n_r]
        self.B_i = B.astype(np.float64)

    def oracle(self, mode=O.GELU_ERF):
        P, Y, Z = O.mlp_shard_fwd(self.X, self.A_i, self.B_i, mode)
        dP, dX, dA, dB = O.mlp_shard_bwd(self.dZ, self.X, self.A_i, self.B_i, mode)
        return dict(P=P, Y=Y, Z=Z, dP=dP, dX=dX, dA_t=dA.T, dB=dB)

    def run_gpu(self, mode=0, accumulate_twice=False, pad_to=8, poison=True, handle=None, sync=True):
        """Runs ntp_mlp_shard_fwd + bwd (on `handle`, else the default one, on torch's current stream); returns
        host float64 arrays plus the raw padded buffers.  sync=False: returns (device tensors, raw) without
        waiting, for callers that overlap several runs."""
        import torch
        import paper_2504_06095_amd as N
        M, H, n_r = self.M, self.H, self.n_r
        ld = max(round_up(n_r, pad_to), 8)
        X, At, B, dZ = (to_dev_bf16(b) for b in (self.X_bits, self.At_bits, self.B_bits, self.dZ_bits))
        fill = float("nan") if poison else 0.0
        mk = lambda r, c: torch.full((r, c), fill, dtype=torch.bfloat16, device="cuda")
        P, Y, dP = mk(M, ld), mk(M, ld), mk(M, ld)
        Z, dX = mk(M, H), mk(M, H)
        dA_t = torch.full((n_r, H), fill, dtype=torch.float32, device="cuda")
        dB = torch.full((n_r, H), fill, dtype=torch.float32, device="cuda")
        N.ntp_mlp_shard_fwd(X, At, B, P[:, :n_r], Y[:, :n_r], Z, n_r, mode, handle=handle)
        N.ntp_mlp_shard_bwd(dZ, X, At, B, P[:, :n_r], Y[:, :n_r], dP[:, :n_r], dX, dA_t, dB, n_r, mode, False, handle=handle)
        if accumulate_twice:
            N.ntp_mlp_shard_bwd(dZ, X, At, B, P[:, :n_r], Y[:, :n_r], dP[:, :n_r], dX, dA_t, dB, n_r, mode, True,
                                handle=handle)
        raw = dict(P=P, Y=Y, dP=dP, ld=ld)
        if not sync:
            return dict(P=P[:, :n_r], Y=Y[:, :n_r], Z=Z, dP=dP[:, :n_r], dX=dX, dA_t=dA_t, dB=dB,
                        _keep=(X, At, B, dZ)), raw
        torch.cuda.synchronize()
        out = dict(P=dev_bf16_to_f64(P[:, :n_r]), Y=dev_bf16_to_f64(Y[:, :n_r]), Z=dev_bf16_to_f64(Z),
                   dP=dev_bf16_to_f64(dP[:, :n_r]), dX=dev_bf16_to_f64(dX),
                   dA_t=dA_t.cpu().numpy().astype(np.float64), dB=dB.cpu().numpy().astype(np.float64))
        return out, raw


class AttnCase:
    """Inputs of one attention shard's projections."""

    def __init__(self, M, H, n_q, n_kv, d, tp, rank, seed=0, tag="attn"):
        self.M, self.H = M, H
        self.plan = O.attn_shard_plan(n_q, n_kv, tp, rank)
        self.w_qkv = (self.plan["q_cnt"] + 2 * self.plan["kv_cnt"]) * d
        self.w_o = self.plan["q_cnt"] * d
        self.X_bits, X = I.normal_bf16(seed, f"{tag}.X", (M, H), I.ACT_STD)
        self.C_bits, Cc = I.normal_bf16(seed, f"{tag}.C.{tp}.{rank}", (M, self.w_o), I.ACT_STD)
        self.dZ_bits, dZ = I.normal_bf16(seed, f"{tag}.dZ", (M, H), I.ACT_STD)
        self.dQKV_bits, dQKV = I.normal_bf16(seed, f"{tag}.dQKV.{tp}.{rank}", (M, self.w_qkv), I.ACT_STD)
        self.Wqkv_bits, Wqkv = I.normal_bf16(seed, f"{tag}.Wqkv.{tp}.{rank}", (self.w_qkv, H), I.WEIGHT_STD)
        self.Wo_bits, Wo = I.normal_bf16(seed, f"{tag}.Wo.{tp}.{rank}", (self.w_o, H), I.WEIGHT_STD)
        f = lambda a: a.astype(np.float64)
        self.X, self.C, self.dZ, self.dQKV = f(X), f(Cc), f(dZ), f(dQKV)
        self.Wqkv_i = f(Wqkv).T.copy()  # paper orientation [H x w_qkv]
        self.Wo_i = f(Wo)               # [w_o x H]

    def oracle(self):
        QKV, Z = O.attn_proj_shard_fwd(self.X, self.Wqkv_i, self.C, self.Wo_i)
        dC, dX, dWqkv, dWo = O.attn_proj_shard_bwd(self.dZ, self.dQKV, self.X, self.C, self.Wqkv_i, self.Wo_i)
        return dict(QKV=QKV, Z=Z, dC=dC, dX=dX, dWqkv=dWqkv.T, dWo=dWo)

    def run_gpu(self):
        import torch
        import paper_2504_06095_amd as N
        M, H, wq, wo = self.M, self.H, self.w_qkv, self.w_o
        X, Cc, dZ, dQKV, Wqkv, Wo = (to_dev_bf16(b) for b in (self.X_bits, self.C_bits, self.dZ_bits,
                                                               self.dQKV_bits, self.Wqkv_bits, self.Wo_bits))
        nan = float("nan")
        mk = lambda r, c: torch.full((r, c), nan, dtype=torch.bfloat16, device="cuda")
        QKV, Z, dC, dX = mk(M, wq), mk(M, H), mk(M, wo), mk(M, H)
        dWqkv = torch.full((wq, H), nan, dtype=torch.float32, device="cuda")
        dWo = torch.full((wo, H), nan, dtype=torch.float32, device="cuda")
        N.ntp_attn_proj_shard_fwd(M, H, wq, wo, X, Wqkv, QKV, Cc, Wo, Z)
        N.ntp_attn_proj_shard_bwd(M, H, wq, wo, dZ, dQKV, X, Cc, Wqkv, Wo, dC, dX, dWqkv, dWo, False)
        torch.cuda.synchronize()
        return dict(QKV=dev_bf16_to_f64(QKV), Z=dev_bf16_to_f64(Z), dC=dev_bf16_to_f64(dC), dX=dev_bf16_to_f64(dX),
                    dWqkv=dWqkv.cpu().numpy().astype(np.float64), dWo=dWo.cpu().numpy().astype(np.float64))


def apply_segments_on_host(segs, spec_pd, unit, src_shards, dst_shapes, dtype):
    """Carry out a segment list with numpy slicing (for checking the host-side segment builder without a GPU)."""
    dst = [np.zeros(s, dtype=dtype) for s in dst_shapes]
    cover = [np.zeros(s[spec_pd] // unit if unit else 0, dtype=np.int64) for s in dst_shapes]
    for (r, s, su, du, n) in segs:
        a, b = slice(su * unit, (su + n) * unit), slice(du * unit, (du + n) * unit)
        if spec_pd == 0:
            dst[s][b, :] = src_shards[r][a, :]
        else:
            dst[s][:, b] = src_shards[r][:, a]
        cover[s][du:du + n] += 1
    return dst, cover
