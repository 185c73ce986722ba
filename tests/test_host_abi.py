"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its
host logic (plans, sub-shard lists, argument checks) agrees with the oracle.  No kernel runs here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2504_06095_amd as N
from oracle import ntp_oracle as O
from paper_2504_06095_amd import binding as Bd
from tests.helpers import apply_segments_on_host

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ntp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ntp_[a-z_0-9]+)\s*\(", header))
    assert declared == set(Bd.EXPORTS)
    lib = Bd.lib()
    for name in declared:
        assert getattr(lib, name) is not None
    assert N.ntp_version() >= 100
    assert Bd.status_string(0) == "ok" and "align" in Bd.status_string(Bd.NTP_ERR_ALIGNMENT)


def test_shard_plan_matches_oracle_exhaustively():
    for dim in list(range(0, 70)) + [586, 4096, 12000, 49152, 53248]:
        for tp in list(range(1, 41)) + [71, 72]:
            for r in range(tp):
                assert N.ntp_shard_plan(dim, tp, r) == O.shard_plan(dim, tp, r)


def test_shard_plan_errors():
    lib = Bd.lib()
    off, w = C.c_int64(), C.c_int64()
    assert lib.ntp_shard_plan(-1, 2, 0, C.byref(off), C.byref(w)) == Bd.NTP_ERR_INVALID_ARG
    assert lib.ntp_shard_plan(4, 0, 0, C.byref(off), C.byref(w)) == Bd.NTP_ERR_INVALID_ARG
    assert lib.ntp_shard_plan(4, 2, 2, C.byref(off), C.byref(w)) == Bd.NTP_ERR_INVALID_ARG
    assert lib.ntp_shard_plan(4, 2, -1, C.byref(off), C.byref(w)) == Bd.NTP_ERR_INVALID_ARG
    assert lib.ntp_shard_plan(4, 2, 0, None, C.byref(w)) == Bd.NTP_ERR_INVALID_ARG
    with pytest.raises(N.NtpError):
        N.ntp_shard_plan(4, 2, 5)


def test_attn_plan_matches_oracle():
    for n_q, n_kv in [(64, 8), (128, 8), (96, 96), (8, 2), (4, 1), (32, 4)]:
        for tp in [1, 2, 3, 5, 7, 8, 30, 32, 71, 72]:
            for r in range(tp):
                got = N.ntp_attn_shard_plan(n_q, n_kv, 128, tp, r)
                want = O.attn_shard_plan(n_q, n_kv, tp, r)
                assert {k: got[k] for k in want} == want
                assert got["w_qkv"] == (want["q_cnt"] + 2 * want["kv_cnt"]) * 128
                assert got["w_o"] == want["q_cnt"] * 128
    with pytest.raises(N.NtpError):
        N.ntp_attn_shard_plan(6, 4, 128, 2, 0)


def test_segments_reproduce_paper_example():
    # Sec. 3.1: hidden 12K, TP32 vs TP30 -> sub-shards of 375 and 25
    segs = N.ntp_reshard_segments(N.tensor_spec(12000, 8, 0), 30, 32)
    assert segs[0] == (0, 0, 0, 0, 375) and segs[1] == (0, 1, 375, 0, 25)
    want = sorted(O.overlap_segments(12000, 30, 32))
    got = sorted((r, s, O.shard_plan(12000, 30, r)[0] + su, n) for (r, s, su, du, n) in segs)
    assert got == want


@pytest.mark.parametrize("pd", [0, 1])
@pytest.mark.parametrize("kind", ["plain", "gqa"])
def test_segments_carried_out_on_host_equal_oracle_reshard(pd, kind):
    rng = np.random.default_rng(0)
    if kind == "plain":
        cases = [(37, 1, 7, 8), (37, 1, 8, 7), (64, 4, 30, 32), (5, 2, 8, 3), (12, 1, 4, 4), (71, 3, 71, 72)]
    else:
        cases = [((8, 2), 3, 3, 4), ((8, 2), 3, 8, 5), ((16, 4), 2, 6, 7), ((4, 1), 5, 2, 4), ((12, 12), 2, 5, 7)]
    for nu, unit, a, b in cases:
        n_q = n_kv = 0
        k = O.PLAIN
        if kind == "gqa":
            (n_q, n_kv), k = nu, O.QKV_GQA
            nu = n_q + 2 * n_kv
        other = 5
        shape = (nu * unit, other) if pd == 0 else (other, nu * unit)
        G = rng.integers(0, 2 ** 32, size=shape, dtype=np.uint32)
        src = [O.cut_shard(G, pd, unit, k, a, r, n_q, n_kv) for r in range(a)]
        want = O.reshard(src, pd, unit, k, a, b, nu, n_q, n_kv)
        spec = N.tensor_spec(shape[0], shape[1], pd, unit, 4, Bd.NTP_KIND_QKV_GQA if kind == "gqa" else Bd.NTP_KIND_PLAIN,
                             n_q, n_kv)
        segs = N.ntp_reshard_segments(spec, a, b)
        got, cover = apply_segments_on_host(segs, pd, unit, src, [w.shape for w in want], np.uint32)
        for s in range(b):
            assert (cover[s] == 1).all()  # every destination unit written exactly once
            assert np.array_equal(got[s], want[s])
        if kind == "plain":
            assert len(segs) <= a + b - 1


def test_segments_at_config_sizes():
    # 405B-shape layer, TP 71 <-> 72: bounded number of sub-shards, full coverage
    for dim, unit in [(53248, 1), (128, 128)]:
        for a, b in [(71, 72), (72, 71)]:
            segs = N.ntp_reshard_segments(N.tensor_spec(dim * unit, 16, 0, unit), a, b)
            assert len(segs) <= a + b - 1
            assert sum(n for *_, n in segs) == dim
    spec = N.tensor_spec(16, (128 + 16) * 128, 1, 128, 4, Bd.NTP_KIND_QKV_GQA, 128, 8)
    segs = N.ntp_reshard_segments(spec, 71, 72)
    per_dst = {}
    for r, s, su, du, n in segs:
        per_dst[s] = per_dst.get(s, 0) + n
    for s in range(72):
        p = O.attn_shard_plan(128, 8, 72, s)
        assert per_dst[s] == p["q_cnt"] + 2 * p["kv_cnt"]


def test_reshard_argument_errors_without_launch():
    lib = Bd.lib()
    n = C.c_int64()
    bad = [N.tensor_spec(10, 4, 2), N.tensor_spec(10, 4, 0, 3), N.tensor_spec(10, 4, 0, 1, 3),
           N.tensor_spec(10, 4, 0, 1, 4, 7), N.tensor_spec(10, 4, 0, 1, 4, Bd.NTP_KIND_QKV_GQA, 4, 2),
           N.tensor_spec(-1, 4, 0)]
    for spec in bad:
        assert lib.ntp_reshard_segments(C.byref(spec), 2, 3, None, 0, C.byref(n)) == Bd.NTP_ERR_INVALID_ARG
    ok = N.tensor_spec(10, 4, 0)
    assert lib.ntp_reshard_segments(C.byref(ok), 0, 3, None, 0, C.byref(n)) == Bd.NTP_ERR_INVALID_ARG
    assert lib.ntp_reshard_segments(C.byref(ok), 2, 3, None, 0, None) == Bd.NTP_ERR_INVALID_ARG
    # null arrays are rejected before anything touches the GPU
    h = Bd.default_handle().ptr
    assert lib.ntp_reshard_grad(h, C.byref(ok), 2, 3, None, None, None, None, None) == Bd.NTP_ERR_INVALID_ARG
    assert lib.ntp_reshard_grad(None, C.byref(ok), 2, 3, None, None, None, None, None) == Bd.NTP_ERR_INVALID_ARG


def test_layer_argument_errors_without_launch():
    lib = Bd.lib()
    h = Bd.default_handle().ptr
    shape = Bd.MlpShape(4, 12, 3, 0)  # H not a multiple of 8
    z = [None, 0] * 6
    assert lib.ntp_mlp_shard_fwd(h, C.byref(shape), *z, None) == Bd.NTP_ERR_ALIGNMENT
    shape = Bd.MlpShape(4, 16, 3, 9)  # unknown GeLU mode
    assert lib.ntp_mlp_shard_fwd(h, C.byref(shape), *z, None) == Bd.NTP_ERR_INVALID_ARG
    shape = Bd.MlpShape(4, 16, 3, 0)  # null tensors
    assert lib.ntp_mlp_shard_fwd(h, C.byref(shape), *z, None) == Bd.NTP_ERR_INVALID_ARG
    assert lib.ntp_mlp_shard_fwd(h, None, *z, None) == Bd.NTP_ERR_INVALID_ARG
    assert lib.ntp_mlp_shard_fwd(None, C.byref(shape), *z, None) == Bd.NTP_ERR_INVALID_ARG  # no handle
    ashape = Bd.AttnShape(4, 16, 12, 8)  # w_qkv not a multiple of 8
    assert lib.ntp_attn_proj_shard_fwd(h, C.byref(ashape), *z, None) == Bd.NTP_ERR_ALIGNMENT


def test_set_workspace_checks_its_arguments():
    """No device memory is touched by setting a workspace: only pointer alignment and size are checked."""
    L = Bd.lib()
    h = Bd.ntp_create()
    assert L.ntp_set_workspace(h.ptr, None, 0) == 0
    assert L.ntp_set_workspace(h.ptr, None, 16) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_set_workspace(h.ptr, 0x1010, 1 << 20) == Bd.NTP_ERR_INVALID_ARG  # not 256-byte aligned
    assert L.ntp_set_workspace(h.ptr, 0x1000, -1) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_set_workspace(None, 0x1000, 256) == Bd.NTP_ERR_INVALID_ARG  # no handle
    assert L.ntp_set_workspace(h.ptr, None, 0) == 0
    Bd.ntp_destroy(h)


def test_handles_are_independent():
    """Workspace and options belong to one handle: what a second handle chooses does not change."""
    a, b = Bd.ntp_create(), Bd.ntp_create()
    assert a.ptr.value != b.ptr.value
    info = Bd.ntp_device_info(a)
    assert info["compute_units"] >= 1 and (info["device"] >= 0 or info["compute_units"] == 256)
    assert Bd.lib().ntp_set_workspace(a.ptr, 0x10000000, 1 << 30) == 0
    skinny = (0, 4096, 640, 8192)  # 48 output tiles of 256 x 256 over K = 8192
    assert Bd.ntp_gemm_choice(*skinny, handle=a)["k_splits"] > 1
    assert Bd.ntp_gemm_choice(*skinny, handle=b)["k_splits"] == 1
    Bd.ntp_set_option(Bd.NTP_OPT_GEMM_TILE, "256x192", handle=b)
    cb = Bd.ntp_gemm_choice(0, 2048, 7022, 12288, handle=b)
    ca = Bd.ntp_gemm_choice(0, 2048, 7022, 12288, handle=a)
    assert (cb["tile_m"], cb["tile_n"]) == (256, 192) and (ca["tile_m"], ca["tile_n"]) == (256, 224)
    Bd.ntp_set_option(Bd.NTP_OPT_GEMM_SPLIT, 1, handle=a)
    assert Bd.ntp_gemm_choice(*skinny, handle=a)["k_splits"] == 1
    Bd.ntp_destroy(a)
    Bd.ntp_destroy(b)
    Bd.ntp_destroy(b)  # destroying twice through the binding is harmless (the pointer is cleared)
    assert Bd.lib().ntp_destroy(None) == 0


def test_set_option_checks_its_arguments():
    L = Bd.lib()
    h = Bd.ntp_create()
    assert L.ntp_set_option(None, Bd.NTP_OPT_GEMM_TILE, 0) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_set_option(h.ptr, -1, 0) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_set_option(h.ptr, 13, 0) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_set_option(h.ptr, Bd.NTP_OPT_GEMM_TILE, 11) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_set_option(h.ptr, Bd.NTP_OPT_GEMM_SPLIT, 9) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_set_option(h.ptr, Bd.NTP_OPT_ATTN_PARTS, 17) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_set_option(h.ptr, Bd.NTP_OPT_RESHARD_NO_TABLE, 2) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_set_option(h.ptr, Bd.NTP_OPT_RESHARD_BLOCK, -4) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_set_option(h.ptr, Bd.NTP_OPT_GEMM_WORKGROUPS, 65537) == Bd.NTP_ERR_INVALID_ARG
    for opt in range(13):
        assert L.ntp_set_option(h.ptr, opt, 1) == 0
        assert L.ntp_set_option(h.ptr, opt, 0) == 0
    Bd.ntp_destroy(h)


def test_workspace_bytes_is_what_an_unlimited_workspace_would_be_used_for():
    """ntp_workspace_bytes: 0 where nothing would be split; otherwise exactly the bytes below which the launcher's
    choice changes (one byte less and the largest split no longer fits)."""
    h = Bd.ntp_create()
    L = Bd.lib()
    # GPT-3 shape MLP shard at TP 7: every GEMM fills the GPU, nothing to split except maybe nothing at all
    big = Bd.MlpShape(2048, 12288, 7022, 0)
    assert Bd.ntp_workspace_bytes(Bd.NTP_CALL_MLP_SHARD, big, handle=h) == 0
    # 405B shape at TP 71: X A_i is 8192 x 750 over K = 16384 -> split; the wish is splits * M * round_up(N64, 16) * 4
    skinny = Bd.MlpShape(8192, 16384, 750, 0)
    need = Bd.ntp_workspace_bytes(Bd.NTP_CALL_MLP_SHARD, skinny, handle=h)
    assert need > 0 and need % (8192 * 768 * 4) == 0
    assert L.ntp_set_workspace(h.ptr, 0x10000000, need) == 0
    with_all = Bd.ntp_gemm_choice(0, 8192, 750, 16384, handle=h)
    assert with_all["k_splits"] * 8192 * 768 * 4 <= need and with_all["k_splits"] > 1
    assert L.ntp_set_workspace(h.ptr, 0x10000000, 8192 * 752 * 4 * 2 - 256) == 0  # (ntp_gemm_choice packs rows to 752)
    assert Bd.ntp_gemm_choice(0, 8192, 750, 16384, handle=h)["k_splits"] == 1
    # attention projections of 3 heads at TP 30 (4096 tokens, hidden 8192) and their core
    att = Bd.AttnShape(4096, 8192, 640, 384)
    assert Bd.ntp_workspace_bytes(Bd.NTP_CALL_ATTN_PROJ_SHARD, att, handle=h) > 0
    plan = N.ntp_attn_shard_plan(64, 8, 128, 30, 0)
    core = N.attn_core_shape(1, 4096, plan, 8, True)
    need_core = Bd.ntp_workspace_bytes(Bd.NTP_CALL_ATTN_CORE_SHARD, core, handle=h)
    assert need_core > 0
    assert L.ntp_set_workspace(h.ptr, 0x10000000, need_core) == 0
    c = Bd.ntp_attn_core_choice(core, handle=h)
    assert max(c["fwd_parts"], c["dq_parts"], c["dkv_parts"]) > 1
    many = N.attn_core_shape(4, 4096, N.ntp_attn_shard_plan(96, 96, 128, 7, 0), 1, False)  # 14 heads x 4 sequences: never cut
    assert Bd.ntp_workspace_bytes(Bd.NTP_CALL_ATTN_CORE_SHARD, many, handle=h) == 0
    # errors
    n = C.c_int64()
    assert L.ntp_workspace_bytes(h.ptr, 7, C.byref(big), C.byref(n)) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_workspace_bytes(h.ptr, 0, None, C.byref(n)) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_workspace_bytes(None, 0, C.byref(big), C.byref(n)) == Bd.NTP_ERR_INVALID_ARG
    assert L.ntp_workspace_bytes(h.ptr, 0, C.byref(Bd.MlpShape(4, 12, 3, 0)), C.byref(n)) == Bd.NTP_ERR_INVALID_ARG
    Bd.ntp_destroy(h)


def test_unprepared_reshard_plan_refuses_to_run():
    """ntp_reshard_plan_run never allocates: a plan that was not prepared returns NOT_PREPARED (or, with no
    device visible, NO_DEVICE) after its argument checks and enqueues nothing."""
    comp, sync = N.ntp_comp_sync_plan(12, 4, 3)
    plan = N.ntp_reshard_plan_create(N.tensor_spec(8, 12, 1), 4, comp, 3, sync)
    L = Bd.lib()
    h = Bd.default_handle()
    vp, i64 = C.c_void_p, C.c_int64
    # fake, non-overlapping, aligned shard addresses: nothing dereferences them before the prepared check
    sp = (vp * 4)(*[0x10000000 + 0x10000 * r for r in range(4)])
    sl = (i64 * 4)(*[3] * 4)
    dp = (vp * 3)(*[0x20000000 + 0x10000 * r for r in range(3)])
    dl = (i64 * 3)(*[4] * 3)
    st = L.ntp_reshard_plan_run(h.ptr, plan._h, sp, sl, dp, dl, None)
    assert st in (Bd.NTP_ERR_NOT_PREPARED, Bd.NTP_ERR_NO_DEVICE)
    assert L.ntp_reshard_plan_run(None, plan._h, sp, sl, dp, dl, None) == Bd.NTP_ERR_INVALID_ARG
    plan.destroy()
