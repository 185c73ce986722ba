"""Split-K form of the shard GEMMs (partial sums to a registered workspace, then a reduce kernel with the
epilogue): every layout and epilogue against the oracle, with the K axis cut into 2..5 chunks including
ragged last chunks, and the automatic choice on a skinny column-parallel shape.  On a real MI355X."""
import sys

import numpy as np
import pytest

from paper_2504_06095_amd import binding as K

from tests.helpers import TOL, AttnCase, MlpCase, rel_err

pytestmark = pytest.mark.gpu
MLP_NAMES = ["P", "Y", "Z", "dP", "dX", "dA_t", "dB"]
ATTN_NAMES = ["QKV", "Z", "dC", "dX", "dWqkv", "dWo"]
SPLIT_TILES = ["256x256", "256x192", "192x256", "256x128", "128x256"]


def _say(msg):
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


def _check_all(got, want, names):
    for k in names:
        assert got[k].shape == want[k].shape, k
        assert np.isfinite(got[k]).all(), f"{k}: non-finite output"
        e = rel_err(got[k], want[k])
        assert e <= TOL, f"{k}: rel err {e:.3e} > {TOL}"


@pytest.fixture
def workspace():
    import torch
    import paper_2504_06095_amd as N
    ws = torch.full((96 << 20,), float("nan"), dtype=torch.float32, device="cuda")  # 384 MiB, poisoned
    N.ntp_set_workspace(ws)
    N.ntp_kernel_timing_enable(1)
    N.ntp_kernel_timing_read()
    yield ws
    N.ntp_kernel_timing_enable(0)
    N.ntp_kernel_timing_read()
    N.ntp_set_workspace(None)


def _gemm_names():
    import paper_2504_06095_amd as N
    return [r["name"] for r in N.ntp_kernel_timing_read() if r["name"].startswith("gemm_")]


@pytest.mark.parametrize("splits", [2, 3, 5])
@pytest.mark.parametrize("tile", SPLIT_TILES)
def test_mlp_split_k_every_tile(workspace, opts, tile, splits):
    # H = 1096 = 17 K tiles + 8, n_r = 1171 = 18 K tiles + 19: ragged last chunks in every layout; M = 1100
    _say(f"mlp split-K tile {tile} splits {splits}")
    opts(K.NTP_OPT_GEMM_TILE, tile)
    opts(K.NTP_OPT_GEMM_SPLIT, splits)
    case = MlpCase(1100, 1096, 8197, 7, 0)
    assert case.n_r == 1171
    got, raw = case.run_gpu(accumulate_twice=True)
    names = _gemm_names()
    assert len(names) == 10 and all(n.endswith(f"{tile}k{splits}") for n in names), names
    want = case.oracle()
    want["dA_t"], want["dB"] = 2 * want["dA_t"], 2 * want["dB"]
    _check_all(got, want, MLP_NAMES)
    for name in ("P", "Y", "dP"):
        assert (raw[name][:, 1171:1176].float().cpu().numpy() == 0).all()


@pytest.mark.parametrize("tile", ["256x256", "224x256", "128x256"])
def test_split_k_last_chunk_shorter_than_a_k_tile(workspace, opts, tile):
    """Five chunks of 256 (320) over K = 1032 (1288): the last chunk has 8 values, no whole K tile, in every layout
    (tokens, hidden size and shard width are each the K of some GEMM of the layer)."""
    _say(f"split-K with a last chunk of 8, tile {tile}")
    opts(K.NTP_OPT_GEMM_TILE, tile)
    opts(K.NTP_OPT_GEMM_SPLIT, 5)
    case = MlpCase(1032, 1032, 1288, 1, 0)
    got, _ = case.run_gpu()
    names = _gemm_names()
    assert len(names) == 6 and all(n.endswith(f"{tile}k5") for n in names), names
    _check_all(got, case.oracle(), MLP_NAMES)


@pytest.mark.parametrize("splits", [2, 4])
def test_attn_proj_split_k(workspace, opts, splits):
    _say(f"attention projections split-K splits {splits}")
    opts(K.NTP_OPT_GEMM_SPLIT, splits)
    case = AttnCase(2200, 1544, 32, 4, 64, 3, 1)  # w_qkv = 960, w_o = 704; K tails of 8, 24 and 0
    got = case.run_gpu()
    names = _gemm_names()
    assert len(names) == 6 and all(n.endswith(f"k{splits}") for n in names), names
    _check_all(got, case.oracle(), ATTN_NAMES)


def test_split_k_chosen_for_skinny_shard_only(workspace):
    """No override: a column-parallel shard with 48 output tiles of 256 x 256 and K = 8192 is split; one
    with enough tiles to fill the GPU is not, and neither is anything without a workspace."""
    import paper_2504_06095_amd as N
    _say("split-K automatic choice")
    skinny = MlpCase(4096, 8192, 640 * 3, 3, 0)
    got, _ = skinny.run_gpu()
    names = _gemm_names()
    assert "k" in names[0].split("_")[-1], names  # X A_i: 4096 x 640 over K = 8192
    _check_all(got, skinny.oracle(), MLP_NAMES)
    wide = MlpCase(8192, 1024, 8192, 1, 0)
    wide.run_gpu()
    names = _gemm_names()
    assert "k" not in names[0].split("_")[-1], names  # X A_i: 8192 x 8192, 1024 tiles
    N.ntp_set_workspace(None)
    skinny.run_gpu()
    names = _gemm_names()
    assert all("k" not in n.split("_")[-1] for n in names), names


def test_split_k_skipped_when_workspace_too_small(opts):
    import torch
    import paper_2504_06095_amd as N
    _say("split-K small workspace")
    ws = torch.zeros(1 << 18, dtype=torch.float32, device="cuda")  # 1 MiB: no partial sums fit
    N.ntp_set_workspace(ws)
    N.ntp_kernel_timing_enable(1)
    N.ntp_kernel_timing_read()
    try:
        opts(K.NTP_OPT_GEMM_SPLIT, 2)
        case = MlpCase(1100, 1096, 8197, 7, 0)
        got, _ = case.run_gpu()
        names = _gemm_names()
        assert all("k" not in n.split("_")[-1] for n in names), names
        _check_all(got, case.oracle(), MLP_NAMES)
    finally:
        N.ntp_kernel_timing_enable(0)
        N.ntp_kernel_timing_read()
        N.ntp_set_workspace(None)


def test_automatic_choice_on_seeded_random_shapes(workspace):
    """Eight seeded random layer shapes through the launcher's own choice of tile, chunks and persistence
    (workspace registered, no override): whatever it picks must match the oracle."""
    rng = np.random.default_rng(20250406)
    picked = set()
    for i in range(8):
        M = int(rng.integers(130, 2600))
        H = int(rng.integers(17, 400)) * 8
        n_r = int(rng.integers(130, 1400))
        _say(f"random shape {i}: M={M} H={H} n_r={n_r}")
        case = MlpCase(M, H, n_r, 1, 0, seed=100 + i, tag=f"rnd{i}")
        got, _ = case.run_gpu()
        picked.update(n.split("_", 3)[-1] for n in _gemm_names())
        _check_all(got, case.oracle(), MLP_NAMES)
    _say(f"variants picked: {sorted(picked)}")
    assert len(picked) >= 3


def test_two_handles_on_two_streams_split_concurrently():
    """The gradient sync runs on a second stream beside the backward pass (Sec. 4.1): two handles, each with a
    workspace of its own, enqueue split-K shard calls on two streams with nothing ordering them against each
    other; both results must match the oracle (a shared workspace would mix their partial sums)."""
    import torch
    import paper_2504_06095_amd as N
    _say("two handles, two streams, split-K on both")
    ha, hb = N.ntp_create(), N.ntp_create()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    wsa = torch.full((24 << 20,), float("nan"), dtype=torch.float32, device="cuda")
    wsb = torch.full((24 << 20,), float("nan"), dtype=torch.float32, device="cuda")
    N.ntp_set_workspace(wsa, handle=ha)
    N.ntp_set_workspace(wsb, handle=hb)
    for hd in (ha, hb):
        N.ntp_set_option(K.NTP_OPT_GEMM_SPLIT, 3, handle=hd)
    ca, cb = MlpCase(1100, 1096, 8197, 7, 0, tag="strm.a"), MlpCase(1100, 1096, 8197, 7, 3, seed=5, tag="strm.b")
    assert K.ntp_gemm_choice(0, 1100, ca.n_r, 1096, handle=ha)["k_splits"] == 3
    torch.cuda.synchronize()
    outs = []
    for rep in range(3):  # several rounds, so that the two streams' kernels really interleave
        with torch.cuda.stream(sa):
            ga, _ = ca.run_gpu(handle=ha, sync=False)
        with torch.cuda.stream(sb):
            gb, _ = cb.run_gpu(handle=hb, sync=False)
        outs.append((ga, gb))
    torch.cuda.synchronize()
    wa, wb = ca.oracle(), cb.oracle()
    for ga, gb in outs:
        for got, want in ((ga, wa), (gb, wb)):
            host = {k: got[k].float().cpu().numpy().astype(np.float64) for k in MLP_NAMES}
            _check_all(host, want, MLP_NAMES)
    N.ntp_destroy(ha)
    N.ntp_destroy(hb)
