"""Pins of the oracle's attention core (Eq. 5), its causal form and its gradient: closed forms, invariances
of the softmax, central finite differences, and agreement of the shard-level wrappers with the per-head calls
and with the unsharded layer."""
import math

import numpy as np
import pytest

from oracle import ntp_oracle as O


def _rng(seed):
    return np.random.default_rng(seed)


def test_causal_rows_see_only_the_past():
    g = _rng(1)
    S, d = 7, 4
    Q, K, V = g.standard_normal((S, d)), g.standard_normal((S, d)), g.standard_normal((S, d))
    C = O.attention_core(Q, K, V, causal=True)
    # row t equals the unmasked attention of query t over keys 0..t
    for t in range(S):
        np.testing.assert_allclose(C[t], O.attention_core(Q[t:t + 1], K[:t + 1], V[:t + 1])[0], atol=1e-13)
    np.testing.assert_allclose(C[0], V[0], atol=1e-14)  # the first token attends to itself only
    # a change of a later key or value leaves earlier rows alone
    K2, V2 = K.copy(), V.copy()
    K2[5] += 3.0
    V2[5] -= 2.0
    C2 = O.attention_core(Q, K2, V2, causal=True)
    np.testing.assert_array_equal(C[:5], C2[:5])
    assert np.abs(C[5:] - C2[5:]).max() > 1e-3


def test_softmax_invariances():
    g = _rng(2)
    S, d = 6, 8
    Q, K, V = g.standard_normal((S, d)), g.standard_normal((S, d)), g.standard_normal((S, d))
    C = O.attention_core(Q, K, V)
    # keys and values permuted together: same output (no mask)
    perm = g.permutation(S)
    np.testing.assert_allclose(O.attention_core(Q, K[perm], V[perm]), C, atol=1e-13)
    # a vector added to every key shifts all scores of a row by the same amount: same output
    np.testing.assert_allclose(O.attention_core(Q, K + g.standard_normal((1, d)), V), C, atol=1e-12)
    # outputs are convex combinations of the value rows
    assert (C.max(0) <= V.max(0) + 1e-12).all() and (C.min(0) >= V.min(0) - 1e-12).all()
    # V constant along the sequence -> output is that constant, for both forms
    Vc = np.tile(g.standard_normal((1, d)), (S, 1))
    for causal in (False, True):
        np.testing.assert_allclose(O.attention_core(Q, K, Vc, causal), Vc, atol=1e-13)
    # huge scores do not overflow (row maximum is subtracted)
    assert np.isfinite(O.attention_core(300.0 * Q, 300.0 * K, V)).all()


@pytest.mark.parametrize("causal", [False, True])
def test_lse_is_the_softmax_normaliser(causal):
    g = _rng(8)
    S, d = 6, 4
    Q, K, V = g.standard_normal((S, d)), g.standard_normal((S, d)), g.standard_normal((S, d))
    lse = O.attention_lse(Q, K, causal)
    W = np.exp((Q @ K.T) / math.sqrt(d) - lse[:, None])
    if causal:
        W = np.tril(W)
    np.testing.assert_allclose(W.sum(1), 1.0, atol=1e-13)
    np.testing.assert_allclose(W @ V, O.attention_core(Q, K, V, causal), atol=1e-13)
    # one visible key: the normaliser is that key's score
    np.testing.assert_allclose(O.attention_lse(Q[:1], K[:1]), (Q[:1] @ K[:1].T)[0] / math.sqrt(d), atol=1e-14)


def test_scale_is_one_over_sqrt_d():
    # two keys, scores q.k / sqrt(d): closed-form logistic weight, for d = 4 and d = 16
    for d in (4, 16):
        q = np.zeros((1, d)); q[0, 0] = 3.0
        K = np.zeros((2, d)); K[0, 0] = 2.0
        V = np.zeros((2, d)); V[0, 0] = 1.0; V[1, 1] = 1.0
        w = 1.0 / (1.0 + math.exp(-6.0 / math.sqrt(d)))
        np.testing.assert_allclose(O.attention_core(q, K, V)[0, :2], [w, 1 - w], atol=1e-14)


@pytest.mark.parametrize("causal", [False, True])
def test_gradient_by_central_differences(causal):
    g = _rng(3)
    S, d = 5, 4
    Q, K, V, dO = (g.standard_normal((S, d)) for _ in range(4))
    dQ, dK, dV = O.attention_core_bwd(Q, K, V, dO, causal)
    h = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for idx in [(0, 0), (1, 3), (2, 1), (4, 2), (3, 0)]:
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += h
            Xm[idx] -= h
            args_p = [Xp if n == name else Y for n, Y in (("Q", Q), ("K", K), ("V", V))]
            args_m = [Xm if n == name else Y for n, Y in (("Q", Q), ("K", K), ("V", V))]
            fd = ((O.attention_core(*args_p, causal) - O.attention_core(*args_m, causal)) * dO).sum() / (2 * h)
            assert abs(fd - G[idx]) < 1e-7 * max(1.0, abs(G[idx])), (name, idx)


def test_gradient_structure():
    g = _rng(4)
    S, d = 6, 4
    Q, K, V, dO = (g.standard_normal((S, d)) for _ in range(4))
    # dV of the unmasked core with uniform attention (all keys equal): every value row gets mean of dO rows' sum / S
    Kc = np.tile(K[:1], (S, 1))
    _, _, dV = O.attention_core_bwd(Q, Kc, V, dO)
    np.testing.assert_allclose(dV, np.tile(dO.sum(0) / S, (S, 1)), atol=1e-13)
    # softmax rows sum to one, so a shift of all scores of a row changes nothing: with all keys equal the
    # query only shifts its row, hence dQ = 0
    dQ, _, _ = O.attention_core_bwd(Q, Kc, V, dO)
    np.testing.assert_allclose(dQ, 0.0, atol=1e-13)
    # causal: the last key/value only feeds the last query
    dQc, dKc, dVc = O.attention_core_bwd(Q, K, V, dO, causal=True)
    np.testing.assert_allclose(dQc[0], 0.0, atol=1e-13)  # query 0 sees one key: its softmax is constant in the score
    w = np.exp((Q[-1] @ K.T) / math.sqrt(d)); w /= w.sum()
    np.testing.assert_allclose(dVc[-1], w[-1] * dO[-1], atol=1e-13)


@pytest.mark.parametrize("n_q,n_kv,tp,causal", [(4, 2, 3, False), (6, 6, 4, True), (8, 2, 5, True), (8, 2, 8, False)])
def test_shard_wrappers_match_per_head_calls_and_the_layer(n_q, n_kv, tp, causal):
    g = _rng(7)
    d, H, S, n_seq = 4, 12, 5, 2
    M = S * n_seq
    group = n_q // n_kv
    X = g.standard_normal((M, H))
    Wq, Wk, Wv = g.standard_normal((H, n_q * d)), g.standard_normal((H, n_kv * d)), g.standard_normal((H, n_kv * d))
    Wo = g.standard_normal((n_q * d, H))
    # unsharded layer, sequence by sequence
    Zfull = np.zeros((M, H))
    for s in range(n_seq):
        rows = slice(s * S, (s + 1) * S)
        Q, K, V = X[rows] @ Wq, X[rows] @ Wk, X[rows] @ Wv
        heads = [O.attention_core(Q[:, h * d:(h + 1) * d], K[:, (h // group) * d:(h // group + 1) * d],
                                  V[:, (h // group) * d:(h // group + 1) * d], causal) for h in range(n_q)]
        Zfull[rows] = np.concatenate(heads, axis=1) @ Wo
    Z = np.zeros((M, H))
    for r in range(tp):
        p, Wqkv_i, Wo_i = O.attn_shard_weights(Wq, Wk, Wv, Wo, n_q, n_kv, d, tp, r)
        if p["q_cnt"] == 0:
            continue
        QKV = X @ Wqkv_i
        C = O.attn_core_shard_fwd(QKV, p, group, d, n_seq, causal)
        Z += C @ Wo_i
        # gradient wrapper against finite differences of sum(C * dC) in a few entries of QKV
        dC = g.standard_normal(C.shape)
        dQKV = O.attn_core_shard_bwd(QKV, dC, p, group, d, n_seq, causal)
        for idx in [(0, 0), (M - 1, QKV.shape[1] - 1), (S, p["q_cnt"] * d), (S - 1, (p["q_cnt"] + p["kv_cnt"]) * d)]:
            h = 1e-6
            Ap, Am = QKV.copy(), QKV.copy()
            Ap[idx] += h
            Am[idx] -= h
            fd = ((O.attn_core_shard_fwd(Ap, p, group, d, n_seq, causal) - O.attn_core_shard_fwd(Am, p, group, d, n_seq, causal)) * dC).sum() / (2 * h)
            assert abs(fd - dQKV[idx]) < 1e-6 * max(1.0, abs(dQKV[idx])), (r, idx)
    np.testing.assert_allclose(Z, Zfull, rtol=1e-10, atol=1e-10)
