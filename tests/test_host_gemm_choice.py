"""Host logic of the GEMM launcher (no GPU): which kernel variant and how many K chunks a shard GEMM gets.
Checks properties that must hold for any tuning of the cost table, plus the choices the benchmark
configurations rely on."""
import itertools

import pytest

import paper_2504_06095_amd as N
from paper_2504_06095_amd import binding as Bd

TILES = {(256, 256), (256, 224), (224, 256), (256, 192), (192, 256), (256, 128), (128, 256), (128, 128)}
FAKE_WS = 0x10000000  # an aligned address: registering touches no memory


@pytest.fixture
def workspace_1gib():
    assert Bd.lib().ntp_set_workspace(Bd.default_handle().ptr, FAKE_WS, 1 << 30) == 0
    yield 1 << 30
    assert Bd.lib().ntp_set_workspace(Bd.default_handle().ptr, None, 0) == 0


def _tiles(c, M, N):
    return -(-M // c["tile_m"]) * -(-N // c["tile_n"])


def test_choice_is_well_formed_over_a_grid_of_shapes():
    for layout, M, Nn, K in itertools.product((0, 1, 2), (1, 100, 586, 2048, 7022), (8, 640, 1792, 12288), (0, 8, 750, 2048, 16384)):
        c = N.ntp_gemm_choice(layout, M, Nn, K)
        assert (c["tile_m"], c["tile_n"]) in TILES and c["wavefronts"] in (4, 8)
        assert c["k_splits"] == 1, "nothing is split without a workspace"
        if not c["ring"]:
            assert (c["tile_m"], c["tile_n"], c["wavefronts"], c["persistent"]) == (128, 128, 4, 0)
        if K < 128 or M * Nn < 2 * 128 * 128:
            assert not c["ring"], (layout, M, Nn, K)


def test_benchmark_configuration_choices():
    # config 2 (GPT-3 shape, TP 7 rank 0): one round of 256 x 224 tiles for fc1, two of 256 x 192 for fc2
    assert _tiles(N.ntp_gemm_choice(0, 2048, 7022, 12288), 2048, 7022) == 256
    c = N.ntp_gemm_choice(1, 2048, 12288, 7022)
    assert (c["tile_m"], c["tile_n"], c["persistent"]) == (256, 192, 1) and _tiles(c, 2048, 12288) == 512
    # the 256 x 256 weight-gradient tile is the non-persistent one
    c = N.ntp_gemm_choice(2, 5376, 12288, 2048)
    assert (c["tile_m"], c["tile_n"], c["persistent"]) == (256, 256, 0)
    # a lone small tile set runs on 8 wavefronts per workgroup
    c = N.ntp_gemm_choice(0, 512, 586, 1024)
    assert (c["tile_m"], c["tile_n"], c["wavefronts"], c["ring"]) == (128, 128, 8, 1)


def test_split_k_only_for_skinny_long_k(workspace_1gib):
    # config 3 QKV projection (48 tiles of 256 x 256 over K = 8192), config 4 fc1, config 2 dC: split
    for (M, Nn, K) in [(4096, 640, 8192), (8192, 750, 16384), (2048, 1792, 12288)]:
        c = N.ntp_gemm_choice(0, M, Nn, K)
        assert 2 <= c["k_splits"] <= 8 and c["persistent"] == 0, (M, Nn, K, c)
        assert _tiles(c, M, Nn) * c["k_splits"] <= 2 * 256
        assert c["k_splits"] * M * (-(-Nn // 16) * 16) * 4 <= workspace_1gib
        assert -(-K // 64) // c["k_splits"] >= 8, "chunks of at least 8 K tiles"
    # enough tiles, or short K: never
    for (layout, M, Nn, K) in [(0, 2048, 7022, 12288), (1, 2048, 12288, 7022), (2, 7022, 12288, 2048), (1, 4096, 8192, 384), (0, 4096, 640, 512)]:
        assert N.ntp_gemm_choice(layout, M, Nn, K)["k_splits"] == 1, (layout, M, Nn, K)


def test_split_k_respects_the_workspace_size():
    assert Bd.lib().ntp_set_workspace(Bd.default_handle().ptr, FAKE_WS, 8 << 20) == 0  # 8 MiB: two slices of 4096 x 640 fp32 would need 21 MB
    try:
        assert N.ntp_gemm_choice(0, 4096, 640, 8192)["k_splits"] == 1
    finally:
        assert Bd.lib().ntp_set_workspace(Bd.default_handle().ptr, None, 0) == 0


def test_choice_rejects_bad_arguments():
    for args in [(3, 8, 8, 8), (-1, 8, 8, 8), (0, 0, 8, 8), (0, 8, 0, 8), (0, 8, 8, -1), (0, 1 << 31, 8, 8)]:
        with pytest.raises(N.NtpError):
            N.ntp_gemm_choice(*args)


def test_schedule_choice_and_override():
    """K-contiguous layouts get the ping-pong schedule on the persistent 8-wavefront tiles; the option forces either."""
    h = Bd.ntp_create()
    c = Bd.ntp_gemm_choice(0, 2048, 7022, 12288, handle=h)
    assert c["persistent"] == 1 and c["pingpong"] == 1
    assert Bd.ntp_gemm_choice(1, 2048, 12288, 7022, handle=h)["pingpong"] == 0
    assert Bd.ntp_gemm_choice(1, 8192, 16384, 750, handle=h)["pingpong"] == 1  # row-parallel layout at short K
    c = Bd.ntp_gemm_choice(2, 7022, 12288, 2048, handle=h)  # weight gradient on the 224 x 256 tile: ping-pong too
    assert (c["tile_m"], c["tile_n"], c["pingpong"]) == (224, 256, 1)
    c = Bd.ntp_gemm_choice(2, 1792, 12288, 2048, handle=h)  # ... on the 192 x 256 tile: default schedule
    assert (c["tile_m"], c["tile_n"], c["pingpong"]) == (192, 256, 0)
    assert Bd.ntp_gemm_choice(0, 512, 586, 1024, handle=h)["pingpong"] == 0  # the small 128 x 128 tile has one schedule
    Bd.ntp_set_option(Bd.NTP_OPT_GEMM_SCHEDULE, 1, handle=h)
    assert Bd.ntp_gemm_choice(0, 2048, 7022, 12288, handle=h)["pingpong"] == 0
    Bd.ntp_set_option(Bd.NTP_OPT_GEMM_SCHEDULE, 2, handle=h)
    assert Bd.ntp_gemm_choice(1, 2048, 12288, 7022, handle=h)["pingpong"] == 1
    assert Bd.ntp_gemm_choice(2, 5376, 12288, 2048, handle=h)["pingpong"] == 0  # 256 x 256 weight-gradient tile: non-persistent
    assert Bd.lib().ntp_set_option(h.ptr, Bd.NTP_OPT_GEMM_SCHEDULE, 3) == Bd.NTP_ERR_INVALID_ARG
    Bd.ntp_destroy(h)
