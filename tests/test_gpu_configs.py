"""Parity at the full sizes of the five benchmark configurations, in the launch configurations
bench.py times (automatic tile choice; with the 1 GiB split-K workspace it registers by default, and
without one), on a real MI355X.

Configs 1-4 compare every output element with the float64 oracle (numpy matmul finishes each
in seconds).  Config 5 (20 GB of gradients) checks the round trip bit-for-bit on the device and
sampled elements of the intermediate layout against the oracle's unit map.
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


def test_config5_reshard_stress_full_size():
    import torch
    import paper_2504_06095_amd as N
    K = N.binding
    Hh, F, nq, nkv, d, a, b = I.C5_H, I.C5_FFN, I.C5_NQ, I.C5_NKV, I.C5_D, I.C5_TRED, I.C5_T
    tensors = [  # name, rows, cols, partition_dim, unit, kind
        ("fc1 dA", Hh, F, 1, 1, O.PLAIN), ("fc2 dB", F, Hh, 0, 1, O.PLAIN),
        ("qkv dW", Hh, (nq + 2 * nkv) * d, 1, d, O.QKV_GQA), ("out dW", nq * d, Hh, 0, d, O.PLAIN),
    ]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    rng = np.random.default_rng(0)
    for name, rows, cols, pd, unit, kind in tensors:
        _say(f"config 5: {name} {rows}x{cols} pd={pd} unit={unit} 71->72->71")
        q, kv = (nq, nkv) if kind == O.QKV_GQA else (0, 0)
        n_units = (cols if pd else rows) // unit
        kc = K.NTP_KIND_QKV_GQA if kind == O.QKV_GQA else K.NTP_KIND_PLAIN
        spec = N.tensor_spec(rows, cols, pd, unit, 4, kc, q, kv)

        def alloc(tp, fill):
            out = []
            for r in range(tp):
                wdt = len(O.unit_list(kind, n_units, tp, r, q, kv)) * unit
                t = torch.empty((rows, wdt) if pd else (wdt, cols), dtype=torch.float32, device="cuda")
                if fill:
                    t.normal_(0.0, I.GRAD_STD, generator=gen)
                else:
                    t.fill_(float("nan"))
                out.append(t)
            return out

        # Build the TP-71 shards from ONE logical tensor so that replicated KV heads agree: fill every
        # shard at random, then overwrite replicas with the lowest rank's copy.
        src = alloc(a, True)
        if kind == O.QKV_GQA:
            first = {}
            for r in range(a):
                for lu, u in enumerate(O.unit_list(kind, n_units, a, r, q, kv)):
                    if u in first:
                        r0, l0 = first[u]
                        src[r][:, lu * unit:(lu + 1) * unit] = src[r0][:, l0 * unit:(l0 + 1) * unit]
                    else:
                        first[u] = (r, lu)
        mid, back = alloc(b, False), alloc(a, False)
        N.ntp_reshard_grad(spec, a, b, src, mid)
        N.ntp_reshard_grad(spec, b, a, mid, back)
        torch.cuda.synchronize()
        for r in range(a):
            assert torch.equal(back[r].view(torch.int32), src[r].view(torch.int32)), f"{name}: round trip rank {r}"
        # sampled elements of the TP-72 layout against the oracle's unit map
        for _ in range(400):
            s = int(rng.integers(0, b))
            ids = O.unit_list(kind, n_units, b, s, q, kv)
            lu = int(rng.integers(0, len(ids)))
            r, sl = O.reshard_source_of(kind, n_units, a, b, s, lu, q, kv)
            e = int(rng.integers(0, unit))
            o = int(rng.integers(0, rows if pd else cols))
            if pd:
                gv, sv = mid[s][o, lu * unit + e], src[r][o, sl * unit + e]
            else:
                gv, sv = mid[s][lu * unit + e, o], src[r][sl * unit + e, o]
            assert gv.view(torch.int32).item() == sv.view(torch.int32).item()
        del src, mid, back
        torch.cuda.empty_cache()
