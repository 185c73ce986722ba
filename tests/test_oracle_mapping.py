"""Pins of the oracle's comp / sync rank assignment and mapped reshard (Sec. 3.1 "Shard-mapping
algorithm", Alg. 1; Appendix hook): hand-worked examples, the properties the paper states for the
mapping (one-to-one shard correspondence on the sync ranks, contiguous sync slices, balanced
computation, equal traffic per pair), and the layer algebra on non-contiguous shards (Sec. 3.1:
any column of A may live in any shard as long as the matching row of B does)."""
import os

import numpy as np
import pytest

from oracle import ntp_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "comp_sync_example.txt")


def _golden():
    a, b = [], []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        (b if f[0] == "b" else a).append([int(x) for x in (f[1:] if f[0] == "b" else f)])
    return np.array(a), np.array(b)


def test_hand_worked_examples():
    a, b = _golden()
    comp, sync = O.comp_sync_plan(12, 4, 3)
    assert comp == list(a[:, 1]) and sync == list(a[:, 2])
    assert [u for u, r in enumerate(comp) if r == 3] == [3, 7, 11]
    comp, sync = O.comp_sync_plan(10, 5, 3)
    assert comp == list(b[:, 1]) and sync == list(b[:, 2])


CASES = [(12000, 32, 30), (53248, 72, 71), (49152, 8, 7), (4096, 8, 7), (4096, 8, 5), (64, 8, 6), (100, 7, 3),
         (5, 8, 7), (0, 4, 3), (17, 4, 4), (128, 72, 71)]


@pytest.mark.parametrize("k,t,tr", CASES)
def test_mapping_properties(k, t, tr):
    comp, sync = O.comp_sync_plan(k, t, tr)
    assert len(comp) == len(sync) == k
    # sync ranks: the contiguous even split over t' ranks, i.e. the degraded replica's own shards
    for i in range(tr):
        off, w = O.shard_plan(k, tr, i)
        assert sync[off:off + w] == [i] * w
    # a sync rank computes a prefix of its own slice: exactly k // t units (all of it when nothing is offloaded)
    keep = k // t
    for i in range(tr):
        off, w = O.shard_plan(k, tr, i)
        mine = [u for u in range(k) if comp[u] == i]
        assert mine == list(range(off, off + (w if t == tr else min(keep, w))))
    # offloaded units go to ranks t' .. t-1 only, and never leave their sync slice's owner for syncing
    assert all((c == s) or (tr <= c < t) for c, s in zip(comp, sync))
    if t > tr:
        counts = O.transfer_counts(comp, t, sync, tr)
        off_counts = counts[tr:, :]  # what each offload rank sends to each sync rank
        # "every pairwise connection gets used to send an equal amount of data": equal up to one unit
        for i in range(tr):
            col = off_counts[:, i]
            assert col.max() - col.min() <= 1
        # computation is balanced over the offload ranks up to one unit
        loads = off_counts.sum(axis=1)
        assert loads.max() - loads.min() <= 1
        # and, when t divides k, over all ranks exactly
        if k % t == 0 and k % tr == 0:
            assert [comp.count(r) for r in range(t)] == [k // t] * t


def test_same_degree_is_the_contiguous_plan():
    comp, sync = O.comp_sync_plan(50, 6, 6)
    assert comp == sync
    assert O.units_of_rank(comp, 6) == [O.unit_list(O.PLAIN, 50, 6, r) for r in range(6)]


def test_rejects_bad_arguments():
    for args in [(-1, 4, 3), (10, 3, 4), (10, 4, 0)]:
        with pytest.raises(ValueError):
            O.comp_sync_plan(*args)


@pytest.mark.parametrize("pd", [0, 1])
@pytest.mark.parametrize("k,t,tr,unit", [(12, 4, 3, 1), (60, 8, 5, 1), (20, 5, 3, 4), (7, 8, 7, 2)])
def test_mapped_reshard_against_brute_force_and_round_trip(pd, k, t, tr, unit):
    rng = np.random.default_rng(k * 100 + t)
    other = 9
    shape = (k * unit, other) if pd == 0 else (other, k * unit)
    G = rng.integers(0, 2 ** 32, size=shape, dtype=np.uint32)
    comp, sync = O.comp_sync_plan(k, t, tr)
    src = [O.cut_shard_mapped(G, pd, unit, comp, t, r) for r in range(t)]
    # the comp layout tiles the logical tensor: every element appears in exactly one shard
    assert sum(s.size for s in src) == G.size
    dst = O.reshard_mapped(src, pd, unit, comp, t, sync, tr)
    # definition: the result is the logical tensor cut by the destination layout; the sync layout is
    # the contiguous one, so it also equals the plain contiguous cut
    for s in range(tr):
        assert np.array_equal(dst[s], O.cut_shard_mapped(G, pd, unit, sync, tr, s))
        assert np.array_equal(dst[s], O.cut_shard(G, pd, unit, O.PLAIN, tr, s))
    # element-by-element brute force through the logical index
    src_ids, dst_ids = O.units_of_rank(comp, t), O.units_of_rank(sync, tr)
    for s in range(tr):
        for local, u in enumerate(dst_ids[s]):
            r = comp[u]
            sl = src_ids[r].index(u)
            for e in range(unit):
                a = np.take(dst[s], local * unit + e, axis=pd)
                b = np.take(src[r], sl * unit + e, axis=pd)
                assert np.array_equal(a, b)
    # and back (the post-sync reshard): identity
    back = O.reshard_mapped(dst, pd, unit, sync, tr, comp, t)
    for r in range(t):
        assert np.array_equal(back[r], src[r])


def test_mlp_on_the_comp_layout_sums_to_the_unsharded_layer():
    # Sec. 3.1, Eq. 1-3: non-contiguous column sets of A with the matching rows of B
    rng = np.random.default_rng(3)
    M, H, n, t, tr = 5, 6, 20, 5, 3
    X, A, B, dZ = rng.normal(size=(M, H)), rng.normal(size=(H, n)), rng.normal(size=(n, H)), rng.normal(size=(M, H))
    comp, _ = O.comp_sync_plan(n, t, tr)
    ids = O.units_of_rank(comp, t)
    assert any(np.any(np.diff(i) > 1) for i in ids if len(i) > 1)  # some shard really is non-contiguous
    _, _, Z = O.mlp_unsharded_fwd(X, A, B)
    dX, dA, dB = O.mlp_unsharded_bwd(dZ, X, A, B)
    Zs, dXs = np.zeros_like(Z), np.zeros_like(dX)
    for r in range(t):
        Ai, Bi = A[:, ids[r]], B[ids[r], :]
        Zs += O.mlp_shard_fwd(X, Ai, Bi)[2]
        _, dXi, dAi, dBi = O.mlp_shard_bwd(dZ, X, Ai, Bi)
        dXs += dXi
        assert np.allclose(dAi, dA[:, ids[r]], rtol=1e-12, atol=1e-12)
        assert np.allclose(dBi, dB[ids[r], :], rtol=1e-12, atol=1e-12)
    assert np.allclose(Zs, Z, rtol=1e-12, atol=1e-12) and np.allclose(dXs, dX, rtol=1e-12, atol=1e-12)


def test_transfer_counts_are_the_hook_splits():
    comp, sync = O.comp_sync_plan(12000, 32, 30)
    c = O.transfer_counts(comp, 32, sync, 30)
    assert c.sum() == 12000
    # sync ranks keep 375 units each and receive 25 from the two offload ranks, 12 or 13 from each
    assert all(c[i, i] == 375 for i in range(30))
    assert all(c[30:, i].sum() == 25 and set(c[30:, i]) <= {12, 13} for i in range(30))
    assert list(c[30:, :].sum(axis=1)) == [375, 375]
