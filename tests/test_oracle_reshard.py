"""Pins for the oracle's gradient reshard (CPU only)."""
import numpy as np
import pytest

from oracle import ntp_oracle as O


def _logical(rows, cols, seed=0):
    # distinct integers so that any misplaced element is visible; viewed as opaque 32-bit words
    g = np.random.default_rng(seed)
    return g.permutation(rows * cols).astype(np.uint32).reshape(rows, cols)


def _cut_all(G, pd, unit, kind, tp, n_q=0, n_kv=0):
    return [O.cut_shard(G, pd, unit, kind, tp, r, n_q, n_kv) for r in range(tp)]


@pytest.mark.parametrize("pd", [0, 1])
@pytest.mark.parametrize("unit", [1, 4])
@pytest.mark.parametrize("n_units,a,b", [(29, 7, 8), (29, 8, 7), (12, 3, 4), (5, 8, 3), (30, 30, 32), (16, 4, 4)])
def test_reshard_brute_force_index_map(pd, unit, n_units, a, b):
    other = 6
    shape = (n_units * unit, other) if pd == 0 else (other, n_units * unit)
    G = _logical(*shape)
    src = _cut_all(G, pd, unit, O.PLAIN, a)
    dst = O.reshard(src, pd, unit, O.PLAIN, a, b, n_units)
    # brute force: walk every logical element, find its place in both layouts
    for j in range(n_units * unit):
        u = j // unit
        r = next(r for r in range(a) if O.shard_plan(n_units, a, r)[0] <= u < sum(O.shard_plan(n_units, a, r)))
        s = next(s for s in range(b) if O.shard_plan(n_units, b, s)[0] <= u < sum(O.shard_plan(n_units, b, s)))
        jl_src = j - O.shard_plan(n_units, a, r)[0] * unit
        jl_dst = j - O.shard_plan(n_units, b, s)[0] * unit
        for o in range(other):
            if pd == 0:
                assert dst[s][jl_dst, o] == src[r][jl_src, o] == G[j, o]
            else:
                assert dst[s][o, jl_dst] == src[r][o, jl_src] == G[o, j]
    # shapes: shard widths follow the plan
    for s in range(b):
        assert dst[s].shape[pd] == O.shard_plan(n_units, b, s)[1] * unit


@pytest.mark.parametrize("pd", [0, 1])
def test_reshard_equals_cutting_the_logical_tensor(pd):
    G = _logical(120, 6) if pd == 0 else _logical(6, 120)
    for a, b in [(7, 8), (8, 7), (30, 32), (5, 5), (1, 9)]:
        dst = O.reshard(_cut_all(G, pd, 1, O.PLAIN, a), pd, 1, O.PLAIN, a, b, 120)
        for s, want in enumerate(_cut_all(G, pd, 1, O.PLAIN, b)):
            assert np.array_equal(dst[s], want)


def test_reshard_round_trip_and_composition():
    G = _logical(8, 213)
    src = _cut_all(G, 1, 1, O.PLAIN, 8)
    a = 8
    for b in (7, 9, 3):
        mid = O.reshard(src, 1, 1, O.PLAIN, a, b, 213)
        back = O.reshard(mid, 1, 1, O.PLAIN, b, a, 213)
        assert all(np.array_equal(x, y) for x, y in zip(back, src))
    ab = O.reshard(src, 1, 1, O.PLAIN, 8, 7, 213)
    abc = O.reshard(ab, 1, 1, O.PLAIN, 7, 5, 213)
    ac = O.reshard(src, 1, 1, O.PLAIN, 8, 5, 213)
    assert all(np.array_equal(x, y) for x, y in zip(abc, ac))
    same = O.reshard(src, 1, 1, O.PLAIN, 8, 8, 213)
    assert all(np.array_equal(x, y) for x, y in zip(same, src))


def test_reshard_preserves_bits():
    # NaN payloads, -0 and denormals travel unchanged (32-bit words, not floats)
    words = np.array([0x7FC00001, 0xFFC12345, 0x80000000, 0x00000001, 0x7F800000, 0x3F800000], dtype=np.uint32)
    G = np.tile(words, (2, 1)).view(np.float32)
    src = _cut_all(G, 1, 1, O.PLAIN, 2)
    dst = O.reshard(src, 1, 1, O.PLAIN, 2, 3, 6)
    got = np.concatenate([d.view(np.uint32) for d in dst], axis=1)
    assert np.array_equal(got, np.tile(words, (2, 1)))


@pytest.mark.parametrize("pd", [0, 1])
def test_reshard_qkv_gqa(pd):
    n_q, n_kv, d, other = 8, 2, 3, 5
    n_units = n_q + 2 * n_kv
    G = _logical(n_units * d, other) if pd == 0 else _logical(other, n_units * d)
    for a, b in [(3, 4), (4, 3), (5, 8), (8, 5), (2, 2)]:
        src = _cut_all(G, pd, d, O.QKV_GQA, a, n_q, n_kv)
        dst = O.reshard(src, pd, d, O.QKV_GQA, a, b, n_units, n_q, n_kv)
        for s, want in enumerate(_cut_all(G, pd, d, O.QKV_GQA, b, n_q, n_kv)):
            assert np.array_equal(dst[s], want)
        back = O.reshard(dst, pd, d, O.QKV_GQA, b, a, n_units, n_q, n_kv)
        assert all(np.array_equal(x, y) for x, y in zip(back, src))


def test_reshard_gqa_reads_lowest_source_rank():
    # KV head 0 is replicated on ranks 0 and 1 (4 query heads, 1 KV head, TP 2); make the
    # replicas differ and check that the destination takes rank 0's copy.
    n_q, n_kv, d = 4, 1, 2
    n_units = 6
    G = _logical(3, n_units * d)
    src = _cut_all(G, 1, d, O.QKV_GQA, 2, n_q, n_kv)
    src[1] = src[1].copy()
    src[1][:, 2 * d:] = 0xDEAD  # rank 1's K and V copies
    dst = O.reshard(src, 1, d, O.QKV_GQA, 2, 4, n_units, n_q, n_kv)
    for s in range(4):
        assert np.array_equal(dst[s][:, d:2 * d], G[:, 4 * d:5 * d])  # K head from the logical tensor
        assert np.array_equal(dst[s][:, 2 * d:], G[:, 5 * d:6 * d])
        assert O.reshard_source_of(O.QKV_GQA, n_units, 2, 4, s, 1, n_q, n_kv) == (0, 2)


def test_reshard_source_of_agrees_with_reshard():
    G = _logical(4, 97)
    src = _cut_all(G, 1, 1, O.PLAIN, 7)
    dst = O.reshard(src, 1, 1, O.PLAIN, 7, 8, 97)
    for s in range(8):
        for lu in range(dst[s].shape[1]):
            r, sl = O.reshard_source_of(O.PLAIN, 97, 7, 8, s, lu)
            assert np.array_equal(dst[s][:, lu], src[r][:, sl])


def test_replica_sum_by_hand():
    """4 query heads, 1 KV head, 2 ranks: logical units [q0 q1 q2 q3 | k0 | v0]; each rank holds 2 query heads and a
    copy of k0 and v0.  The copies become the sum of both ranks' blocks; query heads are left alone."""
    a = np.array([[1., 2., 10., 100.]])   # rank 0: q0 q1 k0 v0
    b = np.array([[3., 4., 20., 200.]])   # rank 1: q2 q3 k0 v0
    got = O.replica_sum([a, b], 1, 1, O.QKV_GQA, 2, 6, 4, 1)
    assert np.array_equal(got[0], [[1., 2., 30., 300.]]) and np.array_equal(got[1], [[3., 4., 30., 300.]])
    assert np.array_equal(a, [[1., 2., 10., 100.]])  # inputs untouched
    # a layout without replication, and a PLAIN tensor, come back unchanged
    c = [np.arange(6.).reshape(1, 6)]
    assert np.array_equal(O.replica_sum(c, 1, 1, O.QKV_GQA, 1, 6, 4, 1)[0], c[0])
    p = [np.arange(4.).reshape(4, 1), np.arange(3.).reshape(3, 1)]
    assert all(np.array_equal(x, y) for x, y in zip(O.replica_sum(p, 0, 1, O.PLAIN, 2, 7), p))


@pytest.mark.parametrize("n_q,n_kv,tp,dst_tp", [(8, 2, 3, 4), (16, 4, 7, 8), (64, 8, 30, 32), (12, 12, 5, 7), (4, 1, 4, 2)])
def test_resharded_qkv_gradient_tiles_the_unsharded_gradient(n_q, n_kv, tp, dst_tp):
    """The invariant the reshard of a weight gradient has to keep (Sec. 3.1: gradients are sharded like their
    weights): every rank's dW_qkv,i = X^T dQKV_i, where dQKV_i holds, for a KV head, only what the rank's own query
    heads contribute; after replica_sum and reshard, EVERY destination rank's block of every unit, replicated K/V
    copies included, equals that unit's columns of the unsharded gradient X^T dQKV.  Without replica_sum the K/V
    blocks of a head that several source ranks hold would miss the other holders' contributions."""
    rng = np.random.default_rng(n_q * 100 + tp)
    M, H, d = 5, 6, 2
    group = n_q // n_kv
    X = rng.standard_normal((M, H))
    # per query head h: its own dQ_h and the dK, dV contributions it makes to its KV head (attention core backward
    # per head; arbitrary values here: only linearity matters)
    dQ = rng.standard_normal((n_q, M, d))
    dKc = rng.standard_normal((n_q, M, d))
    dVc = rng.standard_normal((n_q, M, d))
    dK = np.stack([dKc[g * group:(g + 1) * group].sum(0) for g in range(n_kv)])
    dV = np.stack([dVc[g * group:(g + 1) * group].sum(0) for g in range(n_kv)])
    full = X.T @ np.concatenate([np.concatenate(list(dQ), 1), np.concatenate(list(dK), 1), np.concatenate(list(dV), 1)], 1)
    n_units = n_q + 2 * n_kv
    shards = []
    for r in range(tp):
        p = O.attn_shard_plan(n_q, n_kv, tp, r)
        mine = range(p["q_off"], p["q_off"] + p["q_cnt"])
        cols = [dQ[h] for h in mine]
        for contrib in (dKc, dVc):
            for g in range(p["kv_off"], p["kv_off"] + p["kv_cnt"]):
                cols.append(sum((contrib[h] for h in mine if h // group == g), np.zeros((M, d))))
        dQKV_i = np.concatenate(cols, 1) if cols else np.zeros((M, 0))
        shards.append(O.attn_proj_shard_bwd(np.zeros((M, H)), dQKV_i, X, np.zeros((M, p["q_cnt"] * d)),
                                            np.zeros((H, dQKV_i.shape[1])), np.zeros((p["q_cnt"] * d, H)))[2])
    summed = O.replica_sum(shards, 1, d, O.QKV_GQA, tp, n_units, n_q, n_kv)
    out = O.reshard(summed, 1, d, O.QKV_GQA, tp, dst_tp, n_units, n_q, n_kv)
    for s_ in range(dst_tp):
        want = O.cut_shard(full, 1, d, O.QKV_GQA, dst_tp, s_, n_q, n_kv)
        assert np.allclose(out[s_], want, rtol=1e-12, atol=1e-12)
    if n_kv < tp and n_q != n_kv:  # some head is replicated: leaving the sum out must show
        plain = O.reshard(shards, 1, d, O.QKV_GQA, tp, dst_tp, n_units, n_q, n_kv)
        assert any(not np.allclose(plain[s_], O.cut_shard(full, 1, d, O.QKV_GQA, dst_tp, s_, n_q, n_kv)) for s_ in range(dst_tp))
