"""Host side of the shard-mapping entry points against the oracle (no GPU): the comp / sync rank
assignment (Sec. 3.1, Alg. 1) and the plan between two unit -> rank maps (sub-shards, split sizes,
per-unit source table)."""
import numpy as np
import pytest

import paper_2504_06095_amd as N
from oracle import ntp_oracle as O
from paper_2504_06095_amd.binding import NTP_ERR_INVALID_ARG, NTP_KIND_QKV_GQA, NtpError

PLANS = [(12, 4, 3), (10, 5, 3), (12000, 32, 30), (53248, 72, 71), (53248, 72, 64), (7, 3, 3), (0, 4, 2), (5, 8, 1),
         (3, 8, 5), (1000, 8, 7), (4096, 8, 6), (17, 2, 1)]


@pytest.mark.parametrize("k,t,tr", PLANS)
def test_comp_sync_plan_matches_oracle(k, t, tr):
    assert N.ntp_comp_sync_plan(k, t, tr) == O.comp_sync_plan(k, t, tr)


@pytest.mark.parametrize("k,t,tr", [(-1, 4, 3), (8, 3, 4), (8, 4, 0)])
def test_comp_sync_plan_rejects(k, t, tr):
    with pytest.raises(NtpError) as e:
        N.ntp_comp_sync_plan(k, t, tr)
    assert e.value.status == NTP_ERR_INVALID_ARG


def _expand(segs, src_tp, dst_tp):
    """(src_rank, src_local) of every (dst_rank, dst_local) covered by the segment list."""
    out = {}
    for r, s, su, du, n in segs:
        assert 0 <= r < src_tp and 0 <= s < dst_tp and n > 0
        for i in range(n):
            assert (s, du + i) not in out
            out[(s, du + i)] = (r, su + i)
    return out


def _oracle_sources(smap, src_tp, dmap, dst_tp):
    where = {}
    for r, ids in enumerate(O.units_of_rank(smap, src_tp)):
        for local, u in enumerate(ids):
            where[u] = (r, local)
    return {(s, local): where[u] for s, ids in enumerate(O.units_of_rank(dmap, dst_tp)) for local, u in enumerate(ids)}


def _maps(case):
    kind, k, a, b, seed = case
    if kind == "alg1":
        comp, sync = O.comp_sync_plan(k, a, b)
        return comp, a, sync, b
    if kind == "alg1-back":
        comp, sync = O.comp_sync_plan(k, a, b)
        return sync, b, comp, a
    g = np.random.default_rng(seed)
    return [int(x) for x in g.integers(0, a, k)], a, [int(x) for x in g.integers(0, b, k)], b


MAP_CASES = [("alg1", 12, 4, 3, 0), ("alg1-back", 12, 4, 3, 0), ("alg1", 12000, 32, 30, 0), ("alg1-back", 12000, 32, 30, 0),
             ("alg1", 53248, 72, 71, 0), ("alg1", 100, 8, 8, 0), ("random", 200, 5, 3, 1), ("random", 64, 1, 6, 2),
             ("random", 1, 3, 3, 3), ("alg1", 5, 8, 1, 0)]


@pytest.mark.parametrize("case", MAP_CASES, ids=lambda c: f"{c[0]}-{c[1]}-{c[2]}-{c[3]}")
def test_plan_segments_splits_table(case):
    smap, src_tp, dmap, dst_tp = _maps(case)
    k = len(smap)
    plan = N.ntp_reshard_plan_create(N.tensor_spec(8, k * 2, 1, 2, 4), src_tp, smap, dst_tp, dmap)
    want = _oracle_sources(smap, src_tp, dmap, dst_tp)
    segs = plan.ntp_reshard_plan_segments()
    assert _expand(segs, src_tp, dst_tp) == want
    # destination order, and maximal: two neighbours never continue each other on both sides
    assert [(s[1], s[3]) for s in segs] == sorted((s[1], s[3]) for s in segs)
    for p, q in zip(segs, segs[1:]):
        assert not (p[0] == q[0] and p[1] == q[1] and p[2] + p[4] == q[2] and p[3] + p[4] == q[3])
    assert np.array_equal(np.array(plan.ntp_reshard_plan_splits()).reshape(src_tp, dst_tp),
                          O.transfer_counts(smap, src_tp, dmap, dst_tp))
    table = plan.ntp_reshard_plan_table()
    flat = [want[(s, j)] for s, ids in enumerate(O.units_of_rank(dmap, dst_tp)) for j in range(len(ids))]
    assert table == flat
    plan.destroy()
    plan.destroy()  # a second call is harmless


def test_plan_contiguous_maps_reproduce_the_interval_segments():
    # two contiguous even layouts written as maps give the sub-shards of ntp_reshard_segments
    k, a, b = 1000, 7, 8
    smap = [r for r in range(a) for _ in range(O.shard_plan(k, a, r)[1])]
    dmap = [r for r in range(b) for _ in range(O.shard_plan(k, b, r)[1])]
    spec = N.tensor_spec(4, k, 1, 1, 4)
    plan = N.ntp_reshard_plan_create(spec, a, smap, b, dmap)
    assert plan.ntp_reshard_plan_segments() == N.ntp_reshard_segments(spec, a, b)


def test_plan_rejects_bad_arguments():
    spec = N.tensor_spec(4, 12, 1, 1, 4)
    ok = [0] * 12
    for smap, a, dmap, b in [([3] + ok[1:], 3, ok, 3), (ok, 3, [-1] + ok[1:], 3), (ok, 0, ok, 3)]:
        with pytest.raises(NtpError) as e:
            N.ntp_reshard_plan_create(spec, a, smap, b, dmap)
        assert e.value.status == NTP_ERR_INVALID_ARG
    with pytest.raises(NtpError):  # unit does not divide the partitioned extent
        N.ntp_reshard_plan_create(N.tensor_spec(4, 13, 1, 2, 4), 2, ok[:6], 2, ok[:6])
    with pytest.raises(NtpError):  # grouped-query layouts have their own fixed plan
        N.ntp_reshard_plan_create(N.tensor_spec(4, 12, 1, 1, 4, NTP_KIND_QKV_GQA, 8, 2), 2, ok, 2, ok)
    with pytest.raises(NtpError):  # map length differs from the spec's unit count
        N.ntp_reshard_plan_create(N.tensor_spec(4, 12, 1, 1, 4), 2, ok[:5], 2, ok[:5])
