"""CPU float64 oracle for the NTP shard hot path.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use
this module.  The product (the HIP library and its Python binding) never
imports it, and this module imports nothing from the product.

Everything is the plain definition written out with numpy in float64:
a sharded layer is an exact re-association of the unsharded one (Sec. 3.1,
Eq. 1-6), and a reshard is a permutation of elements.  numpy's matmul is
used as a library step; there is no tiling, fusion or reordering here.

Notation (Sec. 3.1): X is the input [M x H]; A [H x n] is column-partitioned
into A_i, B [n x H] is row-partitioned into B_i; t is the full TP degree and
t' the reduced one.  The oracle keeps the paper's orientation of A and B.
All functions take and return float64 arrays unless they move opaque bits.

Every function here is pinned by tests/test_oracle_*.py against values the
paper prints, closed forms, brute force, finite differences or the properties
the paper states for the result; none is "parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

GELU_ERF = 0   # x * Phi(x), the exact form
GELU_TANH = 1  # the tanh approximation


# ----------------------------------------------------------------------------
# Shard plans (Sec. 3.1, last paragraph of "Attention blocks": the partition
# dimension may not divide evenly; units are split as evenly as possible and
# the remainder goes to the lowest ranks).
# ----------------------------------------------------------------------------
def shard_plan(dim: int, tp: int, rank: int) -> tuple[int, int]:
    """(offset, width) of `rank`'s contiguous slice when `dim` units are split over `tp` ranks."""
    if dim < 0 or tp < 1 or not (0 <= rank < tp):
        raise ValueError("bad shard_plan arguments")
    base, rem = divmod(dim, tp)
    width = base + (1 if rank < rem else 0)
    offset = rank * base + min(rank, rem)
    return offset, width


def attn_shard_plan(n_q: int, n_kv: int, tp: int, rank: int) -> dict:
    """Head-granular plan.  Query heads are the partition unit (Eq. 4-6: the
    W_Q, W_K, W_V, W_O of a head are co-located); with grouped KV heads a rank
    holds every KV head that one of its query heads reads."""
    if n_kv < 1 or n_q % n_kv != 0:
        raise ValueError("n_q must be a multiple of n_kv")
    group = n_q // n_kv
    q_off, q_cnt = shard_plan(n_q, tp, rank)
    if q_cnt == 0:
        return dict(q_off=q_off, q_cnt=0, kv_off=0, kv_cnt=0)
    kv_first = q_off // group
    kv_last = (q_off + q_cnt - 1) // group
    return dict(q_off=q_off, q_cnt=q_cnt, kv_off=kv_first, kv_cnt=kv_last - kv_first + 1)


def overlap_segments(dim: int, src_tp: int, dst_tp: int) -> list[tuple[int, int, int, int]]:
    """Sub-shards made by overlaying two contiguous plans of the same `dim`
    (Sec. 3.1, the paragraph with the hidden-size-12K example).
    Returns (src_rank, dst_rank, first_unit, length) for every non-empty overlap."""
    segs = []
    for r in range(src_tp):
        so, sw = shard_plan(dim, src_tp, r)
        for s in range(dst_tp):
            do, dw = shard_plan(dim, dst_tp, s)
            lo, hi = max(so, do), min(so + sw, do + dw)
            if hi > lo:
                segs.append((r, s, lo, hi - lo))
    return segs


# ----------------------------------------------------------------------------
# GeLU and its derivative.
# ----------------------------------------------------------------------------
def gelu(x: np.ndarray, mode: int = GELU_ERF) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    if mode == GELU_ERF:
        return x * 0.5 * (1.0 + _erf(x / math.sqrt(2.0)))
    if mode == GELU_TANH:
        u = math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)
        return 0.5 * x * (1.0 + np.tanh(u))
    raise ValueError("unknown gelu mode")


def gelu_grad(x: np.ndarray, mode: int = GELU_ERF) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    if mode == GELU_ERF:
        cdf = 0.5 * (1.0 + _erf(x / math.sqrt(2.0)))
        pdf = np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)
        return cdf + x * pdf
    if mode == GELU_TANH:
        c = math.sqrt(2.0 / math.pi)
        u = c * (x + 0.044715 * x ** 3)
        th = np.tanh(u)
        du = c * (1.0 + 3.0 * 0.044715 * x * x)
        return 0.5 * (1.0 + th) + 0.5 * x * (1.0 - th * th) * du
    raise ValueError("unknown gelu mode")


# ----------------------------------------------------------------------------
# MLP block (Eq. 1-3).
# ----------------------------------------------------------------------------
def mlp_unsharded_fwd(X, A, B, mode=GELU_ERF):
    """Eq. 1: Z = GeLU(X A) B.  Returns (P, Y, Z) with P = X A."""
    P = X @ A
    Y = gelu(P, mode)
    return P, Y, Y @ B


def mlp_unsharded_bwd(dZ, X, A, B, mode=GELU_ERF):
    """Gradients of L = sum(Z * dZ) for Eq. 1.  Returns (dX, dA, dB)."""
    P = X @ A
    Y = gelu(P, mode)
    dP = (dZ @ B.T) * gelu_grad(P, mode)
    return dP @ A.T, X.T @ dP, Y.T @ dZ


def mlp_shard_fwd(X, A_i, B_i, mode=GELU_ERF):
    """Eq. 3 then Eq. 2 for one shard: P_i = X A_i, Y_i = GeLU(P_i), Zhat_i = Y_i B_i.
    A_i is [H x n_r] (columns of A), B_i is [n_r x H] (rows of B)."""
    P = X @ A_i
    Y = gelu(P, mode)
    return P, Y, Y @ B_i


def mlp_shard_bwd(dZ, X, A_i, B_i, mode=GELU_ERF):
    """Chain rule on Eq. 2-3 for one shard.  The gradients have the shape and
    partition of A_i / B_i (Sec. 3.1).  Returns (dP_i, dXhat_i, dA_i, dB_i);
    dXhat_i is this shard's partial sum of dX."""
    P = X @ A_i
    Y = gelu(P, mode)
    dY = dZ @ B_i.T
    dP = dY * gelu_grad(P, mode)
    dB = Y.T @ dZ
    dA = X.T @ dP
    dX = dP @ A_i.T
    return dP, dX, dA, dB


# ----------------------------------------------------------------------------
# Attention block: projections (Eq. 4, 6) and the attention core (Eq. 5).
# ----------------------------------------------------------------------------
def attention_core(Q, K, V, causal: bool = False):
    """Eq. 5 for one head: softmax(Q K^T / sqrt(d)) V; Q, K, V are [S x d] (one sequence).  With
    `causal`, query t sees keys 0..t only (the paper writes Attention(Q, K, V) without a mask; decoder
    training masks the future, so both are provided)."""
    d = Q.shape[1]
    S = (Q @ K.T) / math.sqrt(d)
    if causal:
        S = np.where(np.tril(np.ones(S.shape, dtype=bool)), S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    E = np.exp(S)
    return (E / E.sum(axis=1, keepdims=True)) @ V


def attention_lse(Q, K, causal: bool = False):
    """Per query row, log of the sum over the visible keys of exp(q.k / sqrt(d)): the normaliser of Eq. 5's
    softmax, which a forward pass may keep for its backward pass."""
    d = Q.shape[1]
    S = (Q @ K.T) / math.sqrt(d)
    if causal:
        S = np.where(np.tril(np.ones(S.shape, dtype=bool)), S, -np.inf)
    m = S.max(axis=1)
    return m + np.log(np.exp(S - m[:, None]).sum(axis=1))


def attention_core_bwd(Q, K, V, dO, causal: bool = False):
    """Gradients of L = sum(O * dO) for O = attention_core(Q, K, V): chain rule through the softmax.
    Returns (dQ, dK, dV)."""
    d = Q.shape[1]
    S = (Q @ K.T) / math.sqrt(d)
    if causal:
        S = np.where(np.tril(np.ones(S.shape, dtype=bool)), S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    E = np.exp(S)
    P = E / E.sum(axis=1, keepdims=True)
    dV = P.T @ dO
    dP = dO @ V.T
    dS = P * (dP - (dP * P).sum(axis=1, keepdims=True))
    return (dS @ K) / math.sqrt(d), (dS.T @ Q) / math.sqrt(d), dV


def _local_kv_head(plan, group, j):
    """Local KV head read by local query head j of a rank (Sec. 3.1, Eq. 4-6 with grouped KV heads)."""
    return (plan["q_off"] + j) // group - plan["kv_off"]


def attn_core_shard_fwd(QKV, plan, group, d, n_seq, causal=False):
    """Eq. 5 on one rank's local heads: QKV is [M x (q_cnt + 2 kv_cnt) d] with columns
    [Q heads | K heads | V heads] and M = n_seq * S tokens (sequence s = rows s*S .. (s+1)*S-1).
    Returns C [M x q_cnt d], the heads' outputs side by side."""
    M = QKV.shape[0]
    S = M // n_seq
    qc, kc = plan["q_cnt"], plan["kv_cnt"]
    C = np.zeros((M, qc * d))
    for s in range(n_seq):
        rows = slice(s * S, (s + 1) * S)
        for j in range(qc):
            g = _local_kv_head(plan, group, j)
            Q = QKV[rows, j * d:(j + 1) * d]
            K = QKV[rows, (qc + g) * d:(qc + g + 1) * d]
            V = QKV[rows, (qc + kc + g) * d:(qc + kc + g + 1) * d]
            C[rows, j * d:(j + 1) * d] = attention_core(Q, K, V, causal)
    return C


def attn_core_shard_bwd(QKV, dC, plan, group, d, n_seq, causal=False):
    """Gradient of the above with respect to QKV (same layout); a KV head's gradient is the sum over the
    local query heads that read it."""
    M = QKV.shape[0]
    S = M // n_seq
    qc, kc = plan["q_cnt"], plan["kv_cnt"]
    dQKV = np.zeros_like(QKV)
    for s in range(n_seq):
        rows = slice(s * S, (s + 1) * S)
        for j in range(qc):
            g = _local_kv_head(plan, group, j)
            qs, ks, vs = slice(j * d, (j + 1) * d), slice((qc + g) * d, (qc + g + 1) * d), slice((qc + kc + g) * d, (qc + kc + g + 1) * d)
            dQ, dK, dV = attention_core_bwd(QKV[rows, qs], QKV[rows, ks], QKV[rows, vs], dC[rows, qs], causal)
            dQKV[rows, qs] += dQ
            dQKV[rows, ks] += dK
            dQKV[rows, vs] += dV
    return dQKV


def attn_shard_weights(Wq, Wk, Wv, Wo, n_q, n_kv, d, tp, rank):
    """Cut one rank's W_qkv,i [H x (q_cnt + 2 kv_cnt) d] (columns ordered
    [Q heads | K heads | V heads]) and W_O,i [q_cnt d x H] out of the full
    Wq [H x n_q d], Wk, Wv [H x n_kv d], Wo [n_q d x H]."""
    p = attn_shard_plan(n_q, n_kv, tp, rank)
    qs = slice(p["q_off"] * d, (p["q_off"] + p["q_cnt"]) * d)
    ks = slice(p["kv_off"] * d, (p["kv_off"] + p["kv_cnt"]) * d)
    Wqkv_i = np.concatenate([Wq[:, qs], Wk[:, ks], Wv[:, ks]], axis=1)
    return p, Wqkv_i, Wo[qs, :]


def attn_proj_shard_fwd(X, Wqkv_i, C_i, Wo_i):
    """Eq. 6: [Q_i K_i V_i] = X W_qkv,i ; Eq. 4: Zhat_i = C_i W_O,i where C_i is
    the attention output of this rank's heads (an input here)."""
    return X @ Wqkv_i, C_i @ Wo_i


def attn_proj_shard_bwd(dZ, dQKV_i, X, C_i, Wqkv_i, Wo_i):
    """Adjoint of the two projections.  Returns (dC_i, dXhat_i, dWqkv_i, dWo_i)."""
    dC = dZ @ Wo_i.T
    dWo = C_i.T @ dZ
    dX = dQKV_i @ Wqkv_i.T
    dWqkv = X.T @ dQKV_i
    return dC, dX, dWqkv, dWo


def attn_unsharded_fwd(X, Wq, Wk, Wv, Wo, n_q, n_kv, d):
    """Eq. 4-6 for the whole layer with grouped KV heads (query head h reads KV head h // (n_q/n_kv))."""
    group = n_q // n_kv
    Q, K, V = X @ Wq, X @ Wk, X @ Wv
    heads = []
    for h in range(n_q):
        g = h // group
        heads.append(attention_core(Q[:, h * d:(h + 1) * d], K[:, g * d:(g + 1) * d], V[:, g * d:(g + 1) * d]))
    return np.concatenate(heads, axis=1) @ Wo


def attn_shard_layer_fwd(X, Wq, Wk, Wv, Wo, n_q, n_kv, d, tp, rank):
    """One rank's partial sum Zhat_i of the attention layer, going through the
    shard's own projections and the attention core on its local heads."""
    group = n_q // n_kv
    p, Wqkv_i, Wo_i = attn_shard_weights(Wq, Wk, Wv, Wo, n_q, n_kv, d, tp, rank)
    if p["q_cnt"] == 0:
        return np.zeros((X.shape[0], Wo.shape[1]))
    QKV = X @ Wqkv_i
    qw, kw = p["q_cnt"] * d, p["kv_cnt"] * d
    Ql, Kl, Vl = QKV[:, :qw], QKV[:, qw:qw + kw], QKV[:, qw + kw:]
    heads = []
    for j in range(p["q_cnt"]):
        g = (p["q_off"] + j) // group - p["kv_off"]
        heads.append(attention_core(Ql[:, j * d:(j + 1) * d], Kl[:, g * d:(g + 1) * d], Vl[:, g * d:(g + 1) * d]))
    C_i = np.concatenate(heads, axis=1)
    _, Z = attn_proj_shard_fwd(X, Wqkv_i, C_i, Wo_i)
    return Z


# ----------------------------------------------------------------------------
# Gradient reshard (Sec. 3.1 "Shard-mapping algorithm", Appendix hook): both
# layouts are views of one logical tensor partitioned along `partition_dim`
# in units of `unit` elements.
# ----------------------------------------------------------------------------
PLAIN = 0
QKV_GQA = 1


def unit_list(kind, n_units, tp, rank, n_q=0, n_kv=0) -> list[int]:
    """Logical unit ids held by `rank`, in the order they sit in its shard.
    PLAIN: a contiguous range of `n_units`.  QKV_GQA: logical units are
    [n_q Q heads | n_kv K heads | n_kv V heads]; a rank holds its Q heads, then
    the K heads they read, then the same V heads."""
    if kind == PLAIN:
        off, w = shard_plan(n_units, tp, rank)
        return list(range(off, off + w))
    if kind == QKV_GQA:
        if n_units != n_q + 2 * n_kv:
            raise ValueError("n_units must be n_q + 2 n_kv")
        p = attn_shard_plan(n_q, n_kv, tp, rank)
        q = list(range(p["q_off"], p["q_off"] + p["q_cnt"]))
        k = [n_q + g for g in range(p["kv_off"], p["kv_off"] + p["kv_cnt"])]
        v = [n_q + n_kv + g for g in range(p["kv_off"], p["kv_off"] + p["kv_cnt"])]
        return q + k + v
    raise ValueError("unknown kind")


def cut_shard(G, partition_dim, unit, kind, tp, rank, n_q=0, n_kv=0):
    """Cut one rank's shard out of the logical tensor G by fancy indexing."""
    n_units = G.shape[partition_dim] // unit
    ids = unit_list(kind, n_units, tp, rank, n_q, n_kv)
    idx = np.concatenate([np.arange(u * unit, (u + 1) * unit) for u in ids]) if ids else np.zeros(0, dtype=np.int64)
    return np.take(G, idx, axis=partition_dim)


def reshard(src_shards, partition_dim, unit, kind, src_tp, dst_tp, n_units, n_q=0, n_kv=0):
    """Repack shards of the TP=src_tp layout into the TP=dst_tp layout, unit by
    unit: destination unit u of rank s is copied from the lowest source rank
    that holds u.  Moves bits; dtype is whatever the shards carry."""
    where = {}
    for r in range(src_tp):
        for local, u in enumerate(unit_list(kind, n_units, src_tp, r, n_q, n_kv)):
            where.setdefault(u, (r, local))
    out = []
    for s in range(dst_tp):
        ids = unit_list(kind, n_units, dst_tp, s, n_q, n_kv)
        shape = list(src_shards[0].shape)
        shape[partition_dim] = len(ids) * unit
        D = np.empty(shape, dtype=src_shards[0].dtype)
        for local, u in enumerate(ids):
            r, sl = where[u]
            dsl = [slice(None)] * D.ndim
            ssl = [slice(None)] * D.ndim
            dsl[partition_dim] = slice(local * unit, (local + 1) * unit)
            ssl[partition_dim] = slice(sl * unit, (sl + 1) * unit)
            D[tuple(dsl)] = src_shards[r][tuple(ssl)]
        out.append(D)
    return out


def replica_sum(shards, partition_dim, unit, kind, tp, n_units, n_q=0, n_kv=0):
    """Sum of a replicated unit over the ranks that hold it, written back to every holder.

    With grouped KV heads a KV head sits on every rank whose query heads read it
    (attn_shard_plan), and each of those ranks' weight-gradient GEMMs yields only
    the contribution of its own query heads: the gradient of the head is the sum
    of the holders' blocks (chain rule on Eq. 5-6: dW_K,g = sum over the query
    heads h of group g of X^T dK_g^(h)).  Units held by one rank are left alone.
    Returns new float64 shards; the inputs are not modified."""
    holders = {}
    for r in range(tp):
        for local, u in enumerate(unit_list(kind, n_units, tp, r, n_q, n_kv)):
            holders.setdefault(u, []).append((r, local))
    out = [np.array(sh, dtype=np.float64, copy=True) for sh in shards]

    def block(arrs, r, local):
        sl = [slice(None)] * arrs[r].ndim
        sl[partition_dim] = slice(local * unit, (local + 1) * unit)
        return tuple(sl)
    for u, where in holders.items():
        if len(where) < 2:
            continue
        total = np.zeros_like(out[where[0][0]][block(out, *where[0])])
        for r, local in where:  # ascending rank order
            total = total + np.asarray(shards[r], dtype=np.float64)[block(shards, r, local)]
        for r, local in where:
            out[r][block(out, r, local)] = total
    return out


def reshard_source_of(kind, n_units, src_tp, dst_tp, dst_rank, dst_local_unit, n_q=0, n_kv=0):
    """Where one destination unit comes from: (src_rank, src_local_unit).  Used
    to check sampled outputs at sizes where `reshard` itself is too slow."""
    u = unit_list(kind, n_units, dst_tp, dst_rank, n_q, n_kv)[dst_local_unit]
    for r in range(src_tp):
        ids = unit_list(kind, n_units, src_tp, r, n_q, n_kv)
        if u in ids:
            return r, ids.index(u)
    raise AssertionError("unit not held by any source rank")


# ----------------------------------------------------------------------------
# Shard mapping of the healthy replica (Sec. 3.1 "Shard-mapping algorithm",
# Alg. 1 "Comp and Sync Rank Assignment").  The healthy replica computes on all
# t ranks but synchronises on only t' of them (those match the t' shards of a
# degraded replica one to one).  Every partition unit therefore has a rank that
# computes it and a rank that synchronises it.
#
# Reading of the algorithm (its printed form mixes up the two rank counts and
# drops the slice base; the prose fixes what is meant):
#   * sync ranks are ranks 0 .. t'-1 and hold contiguous, even-as-possible
#     slices of the k units (the split of shard_plan(k, t', .));
#   * each sync rank keeps the first k // t units of its slice for its own
#     computation and offloads the rest;
#   * the offloaded units of all sync ranks, taken in unit order, are dealt one
#     by one to the t - t' offload ranks t' .. t-1 in turn, the turn carrying on
#     from one sync rank to the next, so that every (offload rank, sync rank)
#     pair moves the same number of units up to one.
# When t does not divide k the offload ranks absorb the remainder.
# ----------------------------------------------------------------------------
def comp_sync_plan(k: int, t_full: int, t_red: int) -> tuple[list[int], list[int]]:
    """(comp_rank, sync_rank), each a list of k rank numbers."""
    if k < 0 or t_red < 1 or t_full < t_red:
        raise ValueError("need k >= 0 and 1 <= t_red <= t_full")
    comp = [0] * k
    sync = [0] * k
    keep = k // t_full
    n_off = t_full - t_red
    turn = 0
    for i in range(t_red):
        off, w = shard_plan(k, t_red, i)
        for j in range(w):
            u = off + j
            sync[u] = i
            if j < keep or n_off == 0:
                comp[u] = i
            else:
                comp[u] = t_red + turn
                turn = (turn + 1) % n_off
    return comp, sync


def units_of_rank(rank_of_unit, tp: int) -> list[list[int]]:
    """Layout given by a unit -> rank map: rank r holds its units in ascending unit order."""
    out = [[] for _ in range(tp)]
    for u, r in enumerate(rank_of_unit):
        if not (0 <= r < tp):
            raise ValueError("rank out of range")
        out[r].append(u)
    return out


def cut_shard_mapped(G, partition_dim, unit, rank_of_unit, tp, rank):
    """One rank's shard of the logical tensor G under a unit -> rank map."""
    ids = units_of_rank(rank_of_unit, tp)[rank]
    idx = np.concatenate([np.arange(u * unit, (u + 1) * unit) for u in ids]) if ids else np.zeros(0, dtype=np.int64)
    return np.take(G, idx, axis=partition_dim)


def reshard_mapped(src_shards, partition_dim, unit, src_rank_of_unit, src_tp, dst_rank_of_unit, dst_tp):
    """Repack shards between two layouts given by unit -> rank maps, unit by unit
    (the data movement of the pre-sync hook and of the post-sync reshard in the
    Appendix, for the layouts of Alg. 1).  Moves bits."""
    if len(src_rank_of_unit) != len(dst_rank_of_unit):
        raise ValueError("the two maps must cover the same units")
    src_ids = units_of_rank(src_rank_of_unit, src_tp)
    local_in_src = {}
    for r, ids in enumerate(src_ids):
        for local, u in enumerate(ids):
            local_in_src[u] = (r, local)
    out = []
    for s, ids in enumerate(units_of_rank(dst_rank_of_unit, dst_tp)):
        shape = list(src_shards[0].shape)
        shape[partition_dim] = len(ids) * unit
        D = np.empty(shape, dtype=src_shards[0].dtype)
        for local, u in enumerate(ids):
            r, sl = local_in_src[u]
            dsl = [slice(None)] * D.ndim
            ssl = [slice(None)] * D.ndim
            dsl[partition_dim] = slice(local * unit, (local + 1) * unit)
            ssl[partition_dim] = slice(sl * unit, (sl + 1) * unit)
            D[tuple(dsl)] = src_shards[r][tuple(ssl)]
        out.append(D)
    return out


def transfer_counts(src_rank_of_unit, src_tp, dst_rank_of_unit, dst_tp) -> np.ndarray:
    """counts[r][s] = units that move from source rank r to destination rank s: row r is rank r's
    send split, column s is rank s's receive split (the precomputed splits of the Appendix hook)."""
    c = np.zeros((src_tp, dst_tp), dtype=np.int64)
    for r, s in zip(src_rank_of_unit, dst_rank_of_unit):
        c[r, s] += 1
    return c
