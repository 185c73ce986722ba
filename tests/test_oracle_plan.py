"""Pins for the oracle's shard plans and sub-shard lists (CPU only)."""
import os

import numpy as np
import pytest

from oracle import ntp_oracle as O


def _rows(path):
    with open(path) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_plan_brute_force_dealing():
    # Deal units one at a time to ranks 0,1,...,tp-1,0,1,...: the counts are the
    # widths of the most even split with the remainder on the lowest ranks.
    for dim in range(0, 65):
        for tp in range(1, 65):
            counts = [0] * tp
            for u in range(dim):
                counts[u % tp] += 1
            pos = 0
            for r in range(tp):
                off, w = O.shard_plan(dim, tp, r)
                assert w == counts[r]
                assert off == pos
                pos += w
            assert pos == dim


@pytest.mark.parametrize("dim,tp", [(4096, 7), (49152, 7), (49152, 8), (53248, 71), (53248, 72), (12000, 30), (5, 8)])
def test_plan_invariants(dim, tp):
    widths = [O.shard_plan(dim, tp, r)[1] for r in range(tp)]
    offs = [O.shard_plan(dim, tp, r)[0] for r in range(tp)]
    assert sum(widths) == dim
    assert offs == list(np.cumsum([0] + widths[:-1]))
    assert max(widths) - min(widths) <= 1
    assert widths == sorted(widths, reverse=True)


def test_plan_matches_config_list(golden_dir):
    for dim, tp, widest, narrowest in _rows(os.path.join(golden_dir, "config_plans.txt")):
        widths = [O.shard_plan(int(dim), int(tp), r)[1] for r in range(int(tp))]
        assert max(widths) == int(widest) and min(widths) == int(narrowest)
        assert widths[0] == int(widest)


def test_plan_rejects_bad_arguments():
    for args in [(-1, 2, 0), (4, 0, 0), (4, 2, 2), (4, 2, -1)]:
        with pytest.raises(ValueError):
            O.shard_plan(*args)


def test_plan_tp_larger_than_dim():
    widths = [O.shard_plan(3, 5, r)[1] for r in range(5)]
    assert widths == [1, 1, 1, 0, 0]


def test_subshard_example_from_paper(golden_dir):
    (k, n1, n2, big, small), = _rows(os.path.join(golden_dir, "subshard_example.txt"))
    k, n1, n2, big, small = map(int, (k, n1, n2, big, small))
    segs = O.overlap_segments(k, n2, n1)  # src = TP30, dst = TP32
    # TP30 rank 0 holds 400 units: 375 shared with TP32 rank 0, 25 with TP32 rank 1.
    r0 = [(s, ln) for (r, s, _, ln) in segs if r == 0]
    assert r0 == [(0, big), (1, small)]
    # every TP30 shard touches at most 2 TP32 shards (N2 < N1 < 2 N2)
    for r in range(n2):
        assert 1 <= len([1 for sg in segs if sg[0] == r]) <= 2
    assert sum(sg[3] for sg in segs) == k
    assert len(segs) <= n1 + n2 - 1
    # same sub-shards seen from the other side
    back = O.overlap_segments(k, n1, n2)
    assert sorted((s, r, lo, ln) for (r, s, lo, ln) in back) == sorted(segs)


def test_work_ratio_from_paper(golden_dir):
    (t, tr, pct), = _rows(os.path.join(golden_dir, "work_ratio.txt"))
    t, tr, pct = int(t), int(tr), float(pct)
    w_full = O.shard_plan(49152, t, 0)[1]
    w_red = O.shard_plan(49152, tr, 0)[1]
    assert abs((w_red / w_full - 1.0) * 100.0 - pct) < 0.05


def test_segments_cover_every_unit_once():
    for dim, a, b in [(17, 3, 5), (100, 7, 8), (64, 30, 32), (9, 9, 2)]:
        seen = np.zeros(dim, dtype=int)
        for r, s, lo, ln in O.overlap_segments(dim, a, b):
            so, sw = O.shard_plan(dim, a, r)
            do, dw = O.shard_plan(dim, b, s)
            assert so <= lo and lo + ln <= so + sw
            assert do <= lo and lo + ln <= do + dw
            seen[lo:lo + ln] += 1
        assert (seen == 1).all()


# ---- head-granular plan --------------------------------------------------
def test_attn_plan_hand_example():
    # 4 query heads, 2 KV heads (group of 2), 3 ranks: query heads split 2,1,1.
    p = [O.attn_shard_plan(4, 2, 3, r) for r in range(3)]
    assert p[0] == dict(q_off=0, q_cnt=2, kv_off=0, kv_cnt=1)
    assert p[1] == dict(q_off=2, q_cnt=1, kv_off=1, kv_cnt=1)
    assert p[2] == dict(q_off=3, q_cnt=1, kv_off=1, kv_cnt=1)
    assert O.unit_list(O.QKV_GQA, 8, 3, 0, 4, 2) == [0, 1, 4, 6]
    assert O.unit_list(O.QKV_GQA, 8, 3, 1, 4, 2) == [2, 5, 7]
    assert O.unit_list(O.QKV_GQA, 8, 3, 2, 4, 2) == [3, 5, 7]


def test_attn_plan_gqa_config():
    # 64 query heads of 128, 8 KV heads, TP 30: ranks 0-3 hold 3 query heads, the rest 2.
    d = 128
    widths = {}
    for r in range(30):
        p = O.attn_shard_plan(64, 8, 30, r)
        assert p["q_cnt"] == (3 if r < 4 else 2)
        widths[r] = (p["q_cnt"] + 2 * p["kv_cnt"]) * d
        # brute force: the KV heads are exactly the groups of the rank's query heads
        groups = sorted({h // 8 for h in range(p["q_off"], p["q_off"] + p["q_cnt"])})
        assert groups == list(range(p["kv_off"], p["kv_off"] + p["kv_cnt"]))
    assert widths[0] == 640 and widths[2] == 896 and widths[4] == 512
    # rank 2 holds query heads 6,7,8 which straddle KV heads 0 and 1
    assert O.attn_shard_plan(64, 8, 30, 2) == dict(q_off=6, q_cnt=3, kv_off=0, kv_cnt=2)
    for r in range(32):
        p = O.attn_shard_plan(64, 8, 32, r)
        assert (p["q_cnt"], p["kv_cnt"]) == (2, 1)


def test_attn_plan_mha_and_empty_ranks():
    # MHA: every query head has its own KV head.
    for r in range(5):
        p = O.attn_shard_plan(12, 12, 5, r)
        assert (p["kv_off"], p["kv_cnt"]) == (p["q_off"], p["q_cnt"])
    p = O.attn_shard_plan(2, 1, 4, 3)
    assert p["q_cnt"] == 0 and p["kv_cnt"] == 0
    with pytest.raises(ValueError):
        O.attn_shard_plan(6, 4, 2, 0)
