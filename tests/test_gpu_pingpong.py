"""The ping-pong schedule of the ring GEMM kernel (NTP_OPT_GEMM_SCHEDULE = 2) against the oracle: every 8-wavefront
tile shape on ragged shapes (K tails through registers and through the ring, rows and columns past the edge), and
a shape with more output tiles than compute units (workgroups walk over several tiles), and short K with the grid
capped at 8 workgroups (each walks over many output tiles of 1 to 6 K tiles).  On a real MI355X."""
import sys

import numpy as np
import pytest

from paper_2504_06095_amd import binding as K
from tests.helpers import TOL, AttnCase, MlpCase, rel_err

pytestmark = pytest.mark.gpu
TILES = ["256x256", "256x224", "224x256", "256x192", "192x256", "256x128", "128x256"]
MLP_NAMES = ["P", "Y", "Z", "dP", "dX", "dA_t", "dB"]


def _say(msg):
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


def _check_all(got, want, names):
    for k in names:
        assert got[k].shape == want[k].shape, k
        assert np.isfinite(got[k]).all(), f"{k}: non-finite output"
        e = rel_err(got[k], want[k])
        assert e <= TOL, f"{k}: rel err {e:.3e} > {TOL}"


def _pp_names():
    import paper_2504_06095_amd as N
    return [r["name"] for r in N.ntp_kernel_timing_read() if r["name"].startswith("gemm_")]


@pytest.fixture
def pingpong(opts):
    import paper_2504_06095_amd as N
    opts(K.NTP_OPT_GEMM_SCHEDULE, 2)
    N.ntp_kernel_timing_enable(1)
    N.ntp_kernel_timing_read()
    yield
    N.ntp_kernel_timing_enable(0)
    N.ntp_kernel_timing_read()


@pytest.mark.parametrize("pad_to", [8, 64])
@pytest.mark.parametrize("tile", TILES)
def test_mlp_pingpong_every_tile_ragged(pingpong, opts, tile, pad_to):
    # M = 777, H = 1096 = 17 K tiles + 8, n_r = 1001 = 15 K tiles + 41 (pad 64: that tail goes through the ring)
    _say(f"ping-pong mlp tile {tile}, rows padded to {pad_to}")
    opts(K.NTP_OPT_GEMM_TILE, tile)
    case = MlpCase(777, 1096, 2003, 2, 1)
    got, _ = case.run_gpu(pad_to=pad_to)
    names = _pp_names()
    # (the 256 x 256 weight-gradient tile has its own non-persistent form and keeps it)
    assert sum(n.endswith("pp") for n in names) >= (4 if tile == "256x256" else 6), names
    _check_all(got, case.oracle(), MLP_NAMES)


@pytest.mark.parametrize("tile", ["256x256", "224x256", "256x192"])
def test_attn_pingpong(pingpong, opts, tile):
    _say(f"ping-pong attention projections tile {tile}")
    opts(K.NTP_OPT_GEMM_TILE, tile)
    case = AttnCase(520, 1032, 16, 2, 64, 5, 0)
    _check_all(case.run_gpu(), case.oracle(), ["QKV", "Z", "dC", "dX", "dWqkv", "dWo"])


@pytest.mark.parametrize("schedule", [1, 2])
@pytest.mark.parametrize("k_tiles", [1, 2, 3, 5, 6])
def test_few_k_tiles_many_output_tiles_per_workgroup(opts, schedule, k_tiles):
    """One K of the layer = 64 k_tiles and the persistent grid capped at 8 workgroups (NTP_OPT_GEMM_WORKGROUPS): each
    workgroup walks over 5 to 13 output tiles whose K loops are shorter than the ring's look-ahead, under either schedule."""
    kk = 64 * k_tiles
    _say(f"schedule {schedule}, {k_tiles} K tiles per output tile, 8 workgroups")
    opts(K.NTP_OPT_GEMM_SCHEDULE, schedule)
    opts(K.NTP_OPT_GEMM_TILE, "224x256")
    opts(K.NTP_OPT_GEMM_WORKGROUPS, 8)
    # fc1 / dP: K = H; fc2 / dX: K = n_r; dA / dB: K = M -> three cases, each with one short K and longer other sides
    for (M, H, n) in [(1500, kk, 1700), (1500, 1696, kk), (kk, 1504, 1700)]:
        case = MlpCase(M, H, n, 1, 0, tag=f"pp.k{k_tiles}.{M}.{H}")
        got, _ = case.run_gpu(pad_to=64)
        _check_all(got, case.oracle(), MLP_NAMES)


def test_mlp_pingpong_many_tiles_per_workgroup(pingpong):
    """2048 x 12288 x 7022 (the GPT-3-shape shard): 512 to 1536 output tiles per GEMM on 256 compute units, automatic
    tile choice, K = 12288 / 7022 / 2048."""
    from paper_2504_06095_amd import inputs as I
    w = I.C2_MLP
    _say("ping-pong mlp at the GPT-3 shape")
    case = MlpCase(w.M, w.H, w.n, 7, 0, tag=w.name)
    got, _ = case.run_gpu(pad_to=64)
    names = _pp_names()
    assert sum(n.endswith("pp") for n in names) == 6, names
    _check_all(got, case.oracle(), MLP_NAMES)


def test_mlp_pingpong_tiny_extents(pingpong, opts):
    for tile in ("256x256", "224x256"):
        opts(K.NTP_OPT_GEMM_TILE, tile)
        for (M, H, n, tp, rank) in [(1, 8, 3, 3, 0), (3, 72, 17, 1, 0), (65, 64, 64, 1, 0), (300, 136, 200, 1, 0)]:
            _say(f"ping-pong degenerate {tile} M={M} H={H} n={n}")
            case = MlpCase(M, H, n, tp, rank)
            got, _ = case.run_gpu()
            _check_all(got, case.oracle(), MLP_NAMES)
