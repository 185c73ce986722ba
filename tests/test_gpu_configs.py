"""Parity at the full sizes of the five benchmark configurations, in the launch configurations
bench.py times (automatic tile choice; with the 1 GiB split-K workspace it registers by default, and
without one), on a real MI355X.

Configs 1-4 compare every output element with the float64 oracle (numpy matmul finishes each
in seconds).  Config 5 (20 GB of gradients) compares every element of every shard of the TP-72 layout, and of
the round trip, with the oracle's cuts of the same logical tensor (the comparison itself runs on the device).
"""
import sys

import numpy as np
import pytest

from oracle import ntp_oracle as O
from paper_2504_06095_amd import inputs as I
from tests.helpers import TOL, AttnCase, MlpCase, rel_err

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


def _check(got, want, names):
    for k in names:
        assert got[k].shape == want[k].shape, k
        assert np.isfinite(got[k]).all(), f"{k}: non-finite output"
        e = rel_err(got[k], want[k])
        _say(f"    {k}: rel err {e:.2e}")
        assert e <= TOL, f"{k}: rel err {e:.3e} > {TOL}"


MLP_NAMES = ["P", "Y", "Z", "dP", "dX", "dA_t", "dB"]


@pytest.fixture(params=["no workspace", "1 GiB workspace"])
def launch_config(request):
    """bench.py's two launch configurations: nothing registered, or 1 GiB for split-K partial sums."""
    import torch
    import paper_2504_06095_amd as N
    if request.param == "1 GiB workspace":
        N.ntp_set_workspace(torch.full((256 << 20,), float("nan"), dtype=torch.float32, device="cuda"))
    yield request.param
    N.ntp_set_workspace(None)


@pytest.mark.parametrize("w,tp,rank,n_r", [
    (I.C1_MLP, 7, 0, 586),
    (I.C2_MLP, 7, 0, 7022), (I.C2_MLP, 7, 6, 7021), (I.C2_MLP, 8, 0, 6144),
    (I.C4_MLP, 71, 0, 750), (I.C4_MLP, 71, 70, 749), (I.C4_MLP, 72, 0, 740),
])
def test_mlp_config_full_size(launch_config, w, tp, rank, n_r):
    _say(f"{w.name} tp={tp} rank={rank} n_r={n_r}, {launch_config}")
    case = MlpCase(w.M, w.H, w.n, tp, rank, tag=w.name)
    assert case.n_r == n_r
    got, _ = case.run_gpu()
    _check(got, case.oracle(), MLP_NAMES)


@pytest.mark.parametrize("tp,rank,w_qkv,w_o", [(30, 0, 640, 384), (30, 2, 896, 384), (30, 4, 512, 256), (32, 0, 512, 256)])
def test_attn_config_full_size(launch_config, tp, rank, w_qkv, w_o):
    w = I.C3_ATTN
    _say(f"{w.name} tp={tp} rank={rank}, {launch_config}")
    case = AttnCase(w.M, w.H, w.n_q, w.n_kv, w.d, tp, rank, tag=w.name)
    assert (case.w_qkv, case.w_o) == (w_qkv, w_o)
    _check(case.run_gpu(), case.oracle(), ["QKV", "Z", "dC", "dX", "dWqkv", "dWo"])


@pytest.mark.parametrize("hidden,rank", [(6144, 0), (6144, 6), (12288, 0), (12288, 6)])
def test_imbalance_sweep_shapes(launch_config, hidden, rank):
    """The second workload's shapes (Sec. 5.1 "Prototype evaluation": hidden 6144 / 12288, FFN 4 x hidden, head
    dimension 128, 4096 tokens), a TP-8 replica degraded to TP 7: the widest rank (0: 3511 / 7022 FFN columns, 7 / 14
    heads) and the narrowest (6: 3510 / 7021 columns, 6 / 13 heads), MLP shard and attention projections, every
    output against the oracle."""
    heads = hidden // 128
    _say(f"imbalance sweep shape hidden={hidden} rank={rank} of TP 7, {launch_config}")
    mlp = MlpCase(4096, hidden, 4 * hidden, 7, rank, tag=f"imb{hidden}")
    assert mlp.n_r == {(6144, 0): 3511, (6144, 6): 3510, (12288, 0): 7022, (12288, 6): 7021}[(hidden, rank)]
    got, _ = mlp.run_gpu()
    _check(got, mlp.oracle(), MLP_NAMES)
    del got
    att = AttnCase(4096, hidden, heads, heads, 128, 7, rank, tag=f"imb{hidden}")
    assert att.plan["q_cnt"] == {(6144, 0): 7, (6144, 6): 6, (12288, 0): 14, (12288, 6): 13}[(hidden, rank)]
    _check(att.run_gpu(), att.oracle(), ["QKV", "Z", "dC", "dX", "dWqkv", "dWo"])


def test_step_attention_projection_shape(launch_config):
    """The attention projections at the benchmark step's own shape: 2048 tokens, hidden 12288, 96 heads of 128, rank 0
    of TP 7 (14 heads: w_qkv 5376, w_o 1792), in both launch configurations (with the workspace dC is split along K)."""
    _say(f"step shape attention projections, {launch_config}")
    att = AttnCase(2048, 12288, 96, 96, 128, 7, 0, tag="step.attn")
    assert (att.w_qkv, att.w_o) == (5376, 1792)
    _check(att.run_gpu(), att.oracle(), ["QKV", "Z", "dC", "dX", "dWqkv", "dWo"])


def test_config1_reshard_after_backward():
    """Config 1 end to end: the dA_t / dB that the GPU backward produced for EVERY rank of TP 7 are
    repacked into the TP 8 layout; the result must equal the unsharded gradient cut at TP 8."""
    import torch
    import paper_2504_06095_amd as N
    w = I.C1_MLP
    _say("config 1: backward of all 7 ranks, then reshard 7 -> 8")
    dA, dB, want_dA, want_dB = [], [], [], []
    for r in range(7):
        case = MlpCase(w.M, w.H, w.n, 7, r, tag=w.name)
        got, _ = case.run_gpu()
        ref = case.oracle()
        dA.append(torch.from_numpy(got["dA_t"].astype(np.float32)).cuda())
        dB.append(torch.from_numpy(got["dB"].astype(np.float32)).cuda())
        want_dA.append(ref["dA_t"])
        want_dB.append(ref["dB"])
    full_dA, full_dB = np.concatenate(want_dA, 0), np.concatenate(want_dB, 0)  # shard blocks tile the full gradient
    spec = N.tensor_spec(w.n, w.H, 0, 1, 4)
    for shards, full in ((dA, full_dA), (dB, full_dB)):
        dst = [torch.zeros(O.shard_plan(w.n, 8, s)[1], w.H, device="cuda") for s in range(8)]
        N.ntp_reshard_grad(spec, 7, 8, shards, dst)
        torch.cuda.synchronize()
        # reshard is bit-exact: the repacked blocks equal the source blocks re-cut
        src_full = np.concatenate([t.cpu().numpy() for t in shards], 0)
        for s in range(8):
            off, wd = O.shard_plan(w.n, 8, s)
            got = dst[s].cpu().numpy()
            assert np.array_equal(got.view(np.uint32), src_full[off:off + wd].view(np.uint32))
            assert rel_err(got, full[off:off + wd]) <= TOL


C5_TENSORS = [  # name, rows, cols, partition_dim, unit, kind
    ("fc1 dA", I.C5_H, I.C5_FFN, 1, 1, O.PLAIN), ("fc2 dB", I.C5_FFN, I.C5_H, 0, 1, O.PLAIN),
    ("qkv dW", I.C5_H, (I.C5_NQ + 2 * I.C5_NKV) * I.C5_D, 1, I.C5_D, O.QKV_GQA),
    ("out dW", I.C5_NQ * I.C5_D, I.C5_H, 0, I.C5_D, O.PLAIN),
]


@pytest.mark.parametrize("tensor", C5_TENSORS, ids=[t[0].replace(" ", "_") for t in C5_TENSORS])
def test_config5_reshard_stress_full_size(tensor):
    """Config 5, every element: the logical gradient G comes from the keyed generator, the TP-71 shards are the
    oracle's cuts of G (so replicated KV heads agree by construction), and after 71 -> 72 EVERY destination shard,
    replicated K/V copies included, must equal the oracle's TP-72 cut of G bit for bit (both layouts are views
    of one logical tensor: that is the definition of the reshard); then 72 -> 71 must give the TP-71 cuts back."""
    import torch
    import paper_2504_06095_amd as N
    K = N.binding
    nq, nkv, a, b = I.C5_NQ, I.C5_NKV, I.C5_TRED, I.C5_T
    for name, rows, cols, pd, unit, kind in [tensor]:
        _say(f"config 5: {name} {rows}x{cols} pd={pd} unit={unit} 71->72->71, all elements")
        q, kv = (nq, nkv) if kind == O.QKV_GQA else (0, 0)
        kc = K.NTP_KIND_QKV_GQA if kind == O.QKV_GQA else K.NTP_KIND_PLAIN
        spec = N.tensor_spec(rows, cols, pd, unit, 4, kc, q, kv)
        G = I.normal_f32(0, "c5." + name, (rows, cols), I.GRAD_STD)

        def cuts(tp):
            """The oracle's shards of G at this TP degree, on the device (bit patterns)."""
            out = []
            for r in range(tp):
                sh = np.ascontiguousarray(O.cut_shard(G, pd, unit, kind, tp, r, q, kv))
                out.append(torch.from_numpy(sh.view(np.int32)).cuda())
            return out

        def blank(like):
            return [torch.full_like(t, 0x7FC00001) for t in like]  # a NaN pattern no input holds

        src, want_mid = cuts(a), cuts(b)
        del G
        mid = blank(want_mid)
        as_f32 = lambda ts: [t.view(torch.float32) for t in ts]
        N.ntp_reshard_grad(spec, a, b, as_f32(src), as_f32(mid))
        torch.cuda.synchronize()
        for s_ in range(b):
            assert mid[s_].shape == want_mid[s_].shape
            assert torch.equal(mid[s_], want_mid[s_]), f"{name}: TP-{b} shard {s_} differs from the oracle's cut"
        del want_mid
        back = blank(src)
        N.ntp_reshard_grad(spec, b, a, as_f32(mid), as_f32(back))
        torch.cuda.synchronize()
        for r in range(a):
            assert torch.equal(back[r], src[r]), f"{name}: round trip rank {r}"
        del src, mid, back
        torch.cuda.empty_cache()
