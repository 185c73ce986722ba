"""ntp_replica_sum on a real MI355X: the gradient of a KV head that several ranks hold is the sum of the holders'
blocks.  Element by element against the oracle, and end to end: every rank's attention-projection backward,
then the sum, then the reshard must tile the unsharded gradient X^T dQKV, replicated copies included."""
import sys

import numpy as np
import pytest

from oracle import ntp_oracle as O
from paper_2504_06095_amd import binding as K
from paper_2504_06095_amd import inputs as I
from tests import helpers as Hh

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


def _dev(arr, pad=0, misalign=0):
    """fp32 array -> device view [r, c] with row stride c + pad, starting `misalign` floats into its buffer."""
    import torch
    r, c = arr.shape
    flat = torch.full((r * (c + pad) + misalign + 8,), float("nan"), dtype=torch.float32, device="cuda")
    view = flat[misalign: misalign + r * (c + pad)].view(r, c + pad)[:, :c]
    view.copy_(torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda())
    return view, flat


@pytest.mark.parametrize("pd,unit,other,n_q,n_kv,tp,pad,misalign", [
    (0, 8, 40, 16, 4, 5, 0, 0), (1, 8, 33, 16, 4, 7, 0, 0), (0, 3, 10, 8, 2, 3, 5, 1), (1, 5, 9, 8, 1, 8, 3, 2),
    (0, 128, 512, 64, 8, 30, 0, 0), (1, 4, 64, 12, 12, 5, 0, 0), (0, 16, 256, 4, 1, 4, 4, 4),
])
def test_replica_sum_matches_oracle(pd, unit, other, n_q, n_kv, tp, pad, misalign):
    import torch
    import paper_2504_06095_amd as N
    _say(f"replica_sum pd={pd} unit={unit} other={other} heads {n_q}/{n_kv} tp={tp} pad={pad} misalign={misalign}")
    n_units = n_q + 2 * n_kv
    shards_np = []
    for r in range(tp):
        w = len(O.unit_list(O.QKV_GQA, n_units, tp, r, n_q, n_kv)) * unit
        shape = (w, other) if pd == 0 else (other, w)
        shards_np.append(I.normal_f32(0, f"rsum.{pd}.{tp}.{r}", shape, 1.0))
    want = O.replica_sum([s.astype(np.float64) for s in shards_np], pd, unit, O.QKV_GQA, tp, n_units, n_q, n_kv)
    pairs = [_dev(s, pad, misalign) for s in shards_np]
    spec = N.tensor_spec(n_units * unit if pd == 0 else other, other if pd == 0 else n_units * unit, pd, unit, 4,
                         K.NTP_KIND_QKV_GQA, n_q, n_kv)
    shards = [p[0] if p[0].numel() else None for p in pairs]
    N.ntp_replica_sum(spec, tp, shards)
    torch.cuda.synchronize()
    first = [p[0].clone() for p in pairs]
    for (view, flat), w, src in zip(pairs, want, shards_np):
        got = view.cpu().numpy().astype(np.float64)
        # fp32 sums of up to tp values against the float64 sum
        assert np.abs(got - w).max() <= 1e-6 * max(1.0, np.abs(w).max()) * tp
        r, c = src.shape
        body = flat[misalign: misalign + r * (c + pad)].view(r, c + pad)
        assert torch.isnan(body[:, c:]).all() and torch.isnan(flat[:misalign]).all()  # pads untouched
    # units with one holder are bit-identical to the input
    for r in range(tp):
        ids = O.unit_list(O.QKV_GQA, n_units, tp, r, n_q, n_kv)
        for lu, u in enumerate(ids):
            alone = sum(u in O.unit_list(O.QKV_GQA, n_units, tp, o, n_q, n_kv) for o in range(tp)) == 1
            if alone:
                sl = (slice(lu * unit, (lu + 1) * unit), slice(None)) if pd == 0 else (slice(None), slice(lu * unit, (lu + 1) * unit))
                assert np.array_equal(first[r].cpu().numpy()[sl], shards_np[r][sl])


def test_replica_sum_is_deterministic_and_skips_absent_ranks():
    import torch
    import paper_2504_06095_amd as N
    _say("replica_sum determinism, absent holder, plain tensors")
    n_q, n_kv, tp, unit, cols = 8, 1, 8, 16, 256  # one KV head on all eight ranks
    n_units = n_q + 2 * n_kv
    spec = N.tensor_spec(n_units * unit, cols, 0, unit, 4, K.NTP_KIND_QKV_GQA, n_q, n_kv)
    src = [I.normal_f32(0, f"rsum.det.{r}", (3 * unit, cols), 1.0) for r in range(tp)]
    runs = []
    for _ in range(2):
        sh = [torch.from_numpy(s).cuda() for s in src]
        N.ntp_replica_sum(spec, tp, sh)
        torch.cuda.synchronize()
        runs.append(sh)
    for a, b in zip(*runs):
        assert torch.equal(a, b)
    # the K and V blocks now agree on every rank, and equal the fp32 sum taken in ascending rank order
    acc = np.zeros((2 * unit, cols), dtype=np.float32)
    for s in src:
        acc = acc + s[unit:]
    for t in runs[0]:
        assert np.array_equal(t.cpu().numpy()[unit:], acc)
    # rank 3 not on this GPU: the others are summed without it and its slot is not touched
    sh = [torch.from_numpy(s).cuda() for s in src]
    sh[3] = None
    N.ntp_replica_sum(spec, tp, sh)
    torch.cuda.synchronize()
    acc = np.zeros((2 * unit, cols), dtype=np.float32)
    for r, s in enumerate(src):
        if r != 3:
            acc = acc + s[unit:]
    assert np.array_equal(sh[0].cpu().numpy()[unit:], acc)
    # a plain tensor has nothing to sum
    plain = [torch.from_numpy(s).cuda() for s in src]
    keep = [t.clone() for t in plain]
    N.ntp_replica_sum(N.tensor_spec(tp * 3 * unit, cols, 0, unit, 4), tp, plain)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(plain, keep))
    # overlapping shards and 2-byte elements are refused
    with pytest.raises(N.NtpError):
        N.ntp_replica_sum(spec, tp, [runs[0][0]] * tp)
    with pytest.raises(N.NtpError):
        N.ntp_replica_sum(N.tensor_spec(n_units * unit, cols, 0, unit, 2, K.NTP_KIND_QKV_GQA, n_q, n_kv), tp, runs[0])


@pytest.mark.parametrize("n_q,n_kv,d,tp,dst_tp", [(16, 4, 32, 5, 7), (8, 2, 64, 8, 3)])
def test_backward_sum_reshard_tiles_the_unsharded_gradient(n_q, n_kv, d, tp, dst_tp):
    """All ranks of a grouped-query attention block on one GPU: ntp_attn_proj_shard_bwd per rank (each rank's
    dQKV_i holds, for a KV head, only its own query heads' contributions), ntp_replica_sum, ntp_reshard_grad;
    every destination shard must equal the oracle's cut of the unsharded X^T dQKV."""
    import torch
    import paper_2504_06095_amd as N
    _say(f"GQA backward -> replica_sum -> reshard, heads {n_q}/{n_kv} x {d}, TP {tp} -> {dst_tp}")
    M, H = 384, 512
    group = n_q // n_kv
    n_units = n_q + 2 * n_kv
    Xb, X = I.normal_bf16(0, "gqa.X", (M, H), 1.0)
    # per query head: dQ and the head's contributions to dK, dV of its KV head (bf16 values)
    per_head = {nm: [I.normal_bf16(0, f"gqa.{nm}.{hh}", (M, d), 1.0) for hh in range(n_q)] for nm in ("dQ", "dKc", "dVc")}
    f64 = lambda pair: pair[1].astype(np.float64)
    full_cols = [f64(per_head["dQ"][hh]) for hh in range(n_q)]
    contrib_sum = {}
    for nm in ("dKc", "dVc"):
        for g in range(n_kv):
            full_cols.append(sum(f64(per_head[nm][hh]) for hh in range(g * group, (g + 1) * group)))
    full = X.astype(np.float64).T @ np.concatenate(full_cols, 1)      # unsharded dW_qkv in the paper's orientation [H x w]
    full_t = np.ascontiguousarray(full.T)                             # library storage [w x H]
    spec = N.tensor_spec(n_units * d, H, 0, d, 4, K.NTP_KIND_QKV_GQA, n_q, n_kv)
    Xd = Hh.to_dev_bf16(Xb)
    shards = []
    for r in range(tp):
        p = O.attn_shard_plan(n_q, n_kv, tp, r)
        mine = list(range(p["q_off"], p["q_off"] + p["q_cnt"]))
        cols = [per_head["dQ"][hh][1] for hh in mine]
        for nm in ("dKc", "dVc"):
            for g in range(p["kv_off"], p["kv_off"] + p["kv_cnt"]):
                part = sum((per_head[nm][hh][1].astype(np.float32) for hh in mine if hh // group == g), np.zeros((M, d), np.float32))
                cols.append(I.bf16_bits_to_f32(I.round_to_bf16_bits(part)))  # what the rank's attention core would hand over
        dQKV_i = np.concatenate(cols, 1)
        wq = dQKV_i.shape[1]
        dQ_dev = Hh.to_dev_bf16(I.round_to_bf16_bits(dQKV_i))
        Wq = torch.zeros(wq, H, dtype=torch.bfloat16, device="cuda")
        dXp = torch.empty(M, H, dtype=torch.bfloat16, device="cuda")
        dW = torch.full((wq, H), float("nan"), dtype=torch.float32, device="cuda")
        N.ntp_attn_proj_shard_bwd(M, H, wq, p["q_cnt"] * d, None, dQ_dev, Xd, None, Wq, None, None, dXp, dW, None)
        shards.append(dW)
    N.ntp_replica_sum(spec, tp, shards)
    dst = [torch.full((len(O.unit_list(O.QKV_GQA, n_units, dst_tp, s_, n_q, n_kv)) * d, H), float("nan"), dtype=torch.float32,
                      device="cuda") for s_ in range(dst_tp)]
    N.ntp_reshard_grad(spec, tp, dst_tp, shards, dst)
    torch.cuda.synchronize()
    for s_ in range(dst_tp):
        want = O.cut_shard(full_t, 0, d, O.QKV_GQA, dst_tp, s_, n_q, n_kv)
        got = dst[s_].cpu().numpy().astype(np.float64)
        # (the per-rank contributions were rounded to bf16 before the GEMM, as an attention core's output would be)
        assert Hh.rel_err(got, want) <= Hh.TOL, s_
