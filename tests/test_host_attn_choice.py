"""Host logic of the attention core launcher (no GPU): rows per wavefront and how many parts the walks are cut into."""
import pytest

import paper_2504_06095_amd as N
from paper_2504_06095_amd import binding as Bd

FAKE_WS = 0x10000000  # an aligned address: registering touches no memory


def _shape(n_q, n_kv, tp, rank, n_seq, S, causal, d=128):
    plan = N.ntp_attn_shard_plan(n_q, n_kv, d, tp, rank)
    return N.attn_core_shape(n_seq, S, plan, n_q // n_kv, causal)


@pytest.fixture
def workspace_1gib():
    assert Bd.lib().ntp_set_workspace(Bd.default_handle().ptr, FAKE_WS, 1 << 30) == 0
    yield
    assert Bd.lib().ntp_set_workspace(Bd.default_handle().ptr, None, 0) == 0


def test_nothing_is_cut_without_a_workspace():
    for args in [(64, 8, 30, 0, 1, 4096, True), (96, 8, 7, 0, 1, 2048, False), (16, 16, 1, 0, 2, 8192, True)]:
        c = N.ntp_attn_core_choice(_shape(*args))
        assert (c["fwd_parts"], c["dq_parts"], c["dkv_parts"]) == (1, 1, 1)
        assert c["fwd_rows_per_wavefront"] in (16, 32)


def test_few_heads_get_cut_walks(workspace_1gib):
    # config 3, rank 0: 3 query heads on 1 KV head, one causal sequence of 4096 tokens (64 tiles, taken in 32 pairs):
    # 96 forward / dQ workgroups with walks of 65 tiles and 32 dK/dV workgroups with walks of 195.  The forward launch is
    # cut towards two workgroups per compute unit, the two backward kernels (one launch) towards one each
    c = N.ntp_attn_core_choice(_shape(64, 8, 30, 0, 1, 4096, True))
    assert c == dict(fwd_rows_per_wavefront=16, fwd_parts=4, dq_parts=2, dkv_parts=8)
    # the same heads without the mask: 192 and 64 workgroups with walks of 64 and 192 tiles
    c = N.ntp_attn_core_choice(_shape(64, 8, 30, 0, 1, 4096, False))
    assert c == dict(fwd_rows_per_wavefront=16, fwd_parts=2, dq_parts=1, dkv_parts=4)
    # ... and at 8192 tokens (384 and 128 workgroups)
    c = N.ntp_attn_core_choice(_shape(64, 8, 30, 0, 1, 8192, False))
    assert (c["fwd_parts"], c["dq_parts"], c["dkv_parts"]) == (1, 1, 2)
    # many heads and tokens: nothing to gain, and the forward kernel takes 32 rows per wavefront
    c = N.ntp_attn_core_choice(_shape(16, 16, 1, 0, 2, 8192, False))
    assert c == dict(fwd_rows_per_wavefront=32, fwd_parts=1, dq_parts=1, dkv_parts=1)


def test_launches_that_fill_the_device_stay_whole(workspace_1gib):
    # 14 heads x 2048 tokens: 448 forward workgroups of 32 tiles each, or 224 of 33 with the causal pairs: parts of 16
    # tiles would not pay; grouped KV heads leave 64 (32) dK/dV workgroups with walks of 7 heads' tiles
    causal = N.ntp_attn_core_choice(_shape(96, 8, 7, 0, 1, 2048, True))
    full = N.ntp_attn_core_choice(_shape(96, 8, 7, 0, 1, 2048, False))
    assert (causal["fwd_parts"], causal["dq_parts"]) == (1, 1)
    assert (full["fwd_parts"], full["dq_parts"]) == (1, 1)
    assert (causal["dkv_parts"], full["dkv_parts"]) == (8, 4)


def test_step_shape_keeps_whole_walks_with_the_dma_kernels(workspace_1gib):
    # 14 query and 14 KV heads x 2048 tokens, causal: 224 workgroups of 33 tiles in all three launches
    c = N.ntp_attn_core_choice(_shape(96, 96, 7, 0, 1, 2048, True))
    assert c == dict(fwd_rows_per_wavefront=16, fwd_parts=1, dq_parts=1, dkv_parts=1)


def test_register_copy_kernels_keep_their_own_rule(workspace_1gib):
    N.ntp_set_option(Bd.NTP_OPT_ATTN_COPY, 1)
    try:
        c = N.ntp_attn_core_choice(_shape(96, 96, 7, 0, 1, 2048, True))
        assert c == dict(fwd_rows_per_wavefront=16, fwd_parts=2, dq_parts=2, dkv_parts=2)
        c = N.ntp_attn_core_choice(_shape(64, 8, 30, 0, 1, 4096, True))
        assert c == dict(fwd_rows_per_wavefront=16, fwd_parts=5, dq_parts=5, dkv_parts=16)
    finally:
        N.ntp_set_option(Bd.NTP_OPT_ATTN_COPY, 0)


def test_short_walks_are_not_cut(workspace_1gib):
    c = N.ntp_attn_core_choice(_shape(8, 2, 3, 0, 1, 200, True))  # 4 key tiles
    assert (c["fwd_parts"], c["dq_parts"]) == (1, 1)


def test_parts_respect_the_workspace_size():
    assert Bd.lib().ntp_set_workspace(Bd.default_handle().ptr, FAKE_WS, 16 << 20) == 0  # 16 MiB
    try:
        c = N.ntp_attn_core_choice(_shape(64, 8, 30, 0, 1, 4096, True))
        # per part: forward 192 workgroups x 64 rows x 132 floats = 6.5 MB, dQ 192 x 64 x 128 floats = 6.3 MB,
        # dK/dV 64 workgroups x 64 rows x 256 floats = 4 MiB
        assert (c["fwd_parts"], c["dq_parts"], c["dkv_parts"]) == (2, 2, 4)
    finally:
        assert Bd.lib().ntp_set_workspace(Bd.default_handle().ptr, None, 0) == 0


def test_choice_rejects_bad_shapes():
    s = _shape(8, 2, 3, 0, 1, 200, True, d=128)
    s.head_dim = 96
    with pytest.raises(N.NtpError):
        N.ntp_attn_core_choice(s)
