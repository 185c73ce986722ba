"""Pins for the oracle's GeLU, MLP shard and attention-projection shard (CPU only)."""
import math
import os

import numpy as np
import pytest

from oracle import ntp_oracle as O


def _rows(path):
    with open(path) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def _rng(seed):
    return np.random.default_rng(seed)


# ---- GeLU ---------------------------------------------------------------------
def test_gelu_exact_against_normal_table(golden_dir):
    for x, phi in _rows(os.path.join(golden_dir, "normal_cdf_table.txt")):
        x, phi = float(x), float(phi)
        assert abs(float(O.gelu(np.array([x]))[0]) - x * phi) < 2e-10


def test_gelu_closed_forms():
    x = np.linspace(-6, 6, 241)
    for mode in (O.GELU_ERF, O.GELU_TANH):
        assert O.gelu(np.array([0.0]), mode)[0] == 0.0
        assert abs(O.gelu_grad(np.array([0.0]), mode)[0] - 0.5) < 1e-15
        np.testing.assert_allclose(O.gelu(x, mode) - O.gelu(-x, mode), x, atol=1e-13)
        np.testing.assert_allclose(O.gelu_grad(x, mode) + O.gelu_grad(-x, mode), 1.0, atol=1e-13)
        assert abs(O.gelu(np.array([30.0]), mode)[0] - 30.0) < 1e-12
        assert abs(O.gelu_grad(np.array([30.0]), mode)[0] - 1.0) < 1e-12
        assert abs(O.gelu(np.array([-30.0]), mode)[0]) < 1e-12


def test_gelu_modes_are_distinguishable():
    e = float(O.gelu(np.array([1.0]), O.GELU_ERF)[0])
    t = float(O.gelu(np.array([1.0]), O.GELU_TANH)[0])
    assert abs(e - 0.8413447461) < 1e-9
    assert 1e-4 < e - t < 2e-4  # the tanh form is about 1.5e-4 low at x = 1
    with pytest.raises(ValueError):
        O.gelu(np.zeros(1), 7)


@pytest.mark.parametrize("mode", [O.GELU_ERF, O.GELU_TANH])
def test_gelu_grad_is_derivative_of_gelu(mode):
    x = np.linspace(-5, 5, 201)
    h = 1e-5
    fd = (O.gelu(x + h, mode) - O.gelu(x - h, mode)) / (2 * h)
    np.testing.assert_allclose(O.gelu_grad(x, mode), fd, atol=1e-9)


# ---- MLP ------------------------------------------------------------------------
def _loops_mlp(X, A, B):
    """Eq. 1 with explicit Python loops and math.erf: independent of numpy's matmul and of the oracle."""
    M, H = X.shape
    n = A.shape[1]
    Z = np.zeros((M, B.shape[1]))
    for m in range(M):
        for j in range(n):
            p = sum(X[m, h] * A[h, j] for h in range(H))
            y = p * 0.5 * (1.0 + math.erf(p / math.sqrt(2.0)))
            for h in range(B.shape[1]):
                Z[m, h] += y * B[j, h]
    return Z


def test_mlp_unsharded_against_python_loops():
    g = _rng(1)
    X, A, B = g.standard_normal((3, 4)), g.standard_normal((4, 7)), g.standard_normal((7, 5))
    _, _, Z = O.mlp_unsharded_fwd(X, A, B)
    np.testing.assert_allclose(Z, _loops_mlp(X, A, B), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("M,H,n,tp", [(5, 8, 21, 4), (6, 16, 64, 7), (4, 8, 24, 8), (3, 4, 3, 5)])
@pytest.mark.parametrize("mode", [O.GELU_ERF, O.GELU_TANH])
def test_mlp_partials_sum_to_unsharded(M, H, n, tp, mode):
    # Eq. 2: Z = sum_i Y_i B_i for any partition, including tp that does not divide n.
    g = _rng(2)
    X, A, B = g.standard_normal((M, H)), g.standard_normal((H, n)) * 0.3, g.standard_normal((n, H)) * 0.3
    dZ = g.standard_normal((M, H))
    P, Y, Z = O.mlp_unsharded_fwd(X, A, B, mode)
    dX, dA, dB = O.mlp_unsharded_bwd(dZ, X, A, B, mode)
    Zs, dXs = np.zeros_like(Z), np.zeros_like(dX)
    dA_t, dB_t = np.full_like(dA, np.nan), np.full_like(dB, np.nan)
    for r in range(tp):
        off, w = O.shard_plan(n, tp, r)
        A_i, B_i = A[:, off:off + w], B[off:off + w, :]
        P_i, Y_i, Z_i = O.mlp_shard_fwd(X, A_i, B_i, mode)
        np.testing.assert_allclose(P_i, P[:, off:off + w], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(Y_i, Y[:, off:off + w], rtol=1e-12, atol=1e-12)
        dP_i, dX_i, dA_i, dB_i = O.mlp_shard_bwd(dZ, X, A_i, B_i, mode)
        assert dA_i.shape == A_i.shape and dB_i.shape == B_i.shape  # gradients shaped like A_i / B_i
        Zs += Z_i
        dXs += dX_i
        dA_t[:, off:off + w] = dA_i
        dB_t[off:off + w, :] = dB_i
    scale = np.abs(Z).max()
    np.testing.assert_allclose(Zs, Z, atol=1e-12 * scale)
    np.testing.assert_allclose(dXs, dX, atol=1e-12 * np.abs(dX).max())
    np.testing.assert_allclose(dA_t, dA, atol=1e-12 * np.abs(dA).max())  # shard blocks tile the full gradient
    np.testing.assert_allclose(dB_t, dB, atol=1e-12 * np.abs(dB).max())


@pytest.mark.parametrize("mode", [O.GELU_ERF, O.GELU_TANH])
def test_mlp_shard_bwd_finite_differences(mode):
    # L = sum(Zhat_i * dZ); central differences on every input entry.
    g = _rng(3)
    M, H, n, tp = 3, 4, 7, 3
    X, A, B = g.standard_normal((M, H)), g.standard_normal((H, n)), g.standard_normal((n, H))
    dZ = g.standard_normal((M, H))
    off, w = O.shard_plan(n, tp, 1)
    A_i, B_i = A[:, off:off + w].copy(), B[off:off + w, :].copy()

    def loss(Xv, Av, Bv):
        return float((O.mlp_shard_fwd(Xv, Av, Bv, mode)[2] * dZ).sum())

    dP, dX, dA, dB = O.mlp_shard_bwd(dZ, X, A_i, B_i, mode)
    h = 1e-6
    for arr, grad, which in ((X, dX, 0), (A_i, dA, 1), (B_i, dB, 2)):
        for idx in np.ndindex(arr.shape):
            args = [X.copy(), A_i.copy(), B_i.copy()]
            args[which][idx] += h
            up = loss(*args)
            args[which][idx] -= 2 * h
            dn = loss(*args)
            assert abs((up - dn) / (2 * h) - grad[idx]) < 1e-7 * max(1.0, abs(grad[idx]))
    # dP is the gradient with respect to the pre-activation: check through Y = gelu(P)
    P, Y, _ = O.mlp_shard_fwd(X, A_i, B_i, mode)
    np.testing.assert_allclose(dP, (dZ @ B_i.T) * O.gelu_grad(P, mode), rtol=1e-13)
    fdP = np.zeros_like(P)
    for idx in np.ndindex(P.shape):
        Pp, Pm = P.copy(), P.copy()
        Pp[idx] += h
        Pm[idx] -= h
        fdP[idx] = (((O.gelu(Pp, mode) @ B_i) * dZ).sum() - ((O.gelu(Pm, mode) @ B_i) * dZ).sum()) / (2 * h)
    np.testing.assert_allclose(dP, fdP, atol=1e-7)


def test_mlp_unsharded_bwd_finite_differences():
    g = _rng(4)
    X, A, B = g.standard_normal((2, 3)), g.standard_normal((3, 5)), g.standard_normal((5, 3))
    dZ = g.standard_normal((2, 3))
    dX, dA, dB = O.mlp_unsharded_bwd(dZ, X, A, B)
    h = 1e-6
    for arr, grad, which in ((X, dX, 0), (A, dA, 1), (B, dB, 2)):
        for idx in np.ndindex(arr.shape):
            args = [X.copy(), A.copy(), B.copy()]
            args[which][idx] += h
            up = (O.mlp_unsharded_fwd(*args)[2] * dZ).sum()
            args[which][idx] -= 2 * h
            dn = (O.mlp_unsharded_fwd(*args)[2] * dZ).sum()
            assert abs((up - dn) / (2 * h) - grad[idx]) < 1e-7 * max(1.0, abs(grad[idx]))


# ---- attention -----------------------------------------------------------------
def test_attention_core_special_cases():
    g = _rng(5)
    V = g.standard_normal((4, 3))
    # all keys equal -> uniform weights -> every output row is the mean of V
    Q = g.standard_normal((5, 3))
    K = np.tile(g.standard_normal((1, 3)), (4, 1))
    np.testing.assert_allclose(O.attention_core(Q, K, V), np.tile(V.mean(0), (5, 1)), atol=1e-13)
    # a single key -> output is that value row
    np.testing.assert_allclose(O.attention_core(Q, K[:1], V[:1]), np.tile(V[:1], (5, 1)), atol=1e-13)
    # one dominant key -> picks its value row; the 1/sqrt(d) scale matters for the 2-key closed form
    q = np.array([[2.0, 0.0, 0.0, 0.0]])
    Kk = np.array([[1.0, 0, 0, 0], [0.0, 0, 0, 0]])
    Vv = np.array([[1.0, 0, 0, 0], [0.0, 1, 0, 0]])
    w = 1.0 / (1.0 + math.exp(-1.0))  # scores 2/sqrt(4)=1 and 0
    np.testing.assert_allclose(O.attention_core(q, Kk, Vv)[0, :2], [w, 1 - w], atol=1e-13)


@pytest.mark.parametrize("n_q,n_kv,tp", [(4, 2, 3), (6, 6, 4), (8, 2, 5), (8, 2, 8), (4, 1, 6)])
def test_attention_partials_sum_to_unsharded(n_q, n_kv, tp):
    # Eq. 4: Z = sum_i MultiHead_i(X) W_O,i for a head-granular partition (with grouped KV heads).
    g = _rng(6)
    M, H, d = 5, 12, 4
    X = g.standard_normal((M, H))
    Wq, Wk, Wv = (g.standard_normal((H, n_q * d)) * 0.4, g.standard_normal((H, n_kv * d)) * 0.4,
                  g.standard_normal((H, n_kv * d)) * 0.4)
    Wo = g.standard_normal((n_q * d, H)) * 0.4
    Z = O.attn_unsharded_fwd(X, Wq, Wk, Wv, Wo, n_q, n_kv, d)
    Zs = sum(O.attn_shard_layer_fwd(X, Wq, Wk, Wv, Wo, n_q, n_kv, d, tp, r) for r in range(tp))
    np.testing.assert_allclose(Zs, Z, atol=1e-12 * np.abs(Z).max())


def test_attn_shard_projection_blocks_equal_unsharded_columns():
    g = _rng(7)
    M, H, d, n_q, n_kv, tp = 4, 8, 2, 8, 2, 3
    X = g.standard_normal((M, H))
    Wq, Wk, Wv = g.standard_normal((H, n_q * d)), g.standard_normal((H, n_kv * d)), g.standard_normal((H, n_kv * d))
    Wo = g.standard_normal((n_q * d, H))
    Q, K, V = X @ Wq, X @ Wk, X @ Wv
    for r in range(tp):
        p, Wqkv_i, Wo_i = O.attn_shard_weights(Wq, Wk, Wv, Wo, n_q, n_kv, d, tp, r)
        C_i = g.standard_normal((M, p["q_cnt"] * d))
        QKV, Zp = O.attn_proj_shard_fwd(X, Wqkv_i, C_i, Wo_i)
        qw, kw = p["q_cnt"] * d, p["kv_cnt"] * d
        np.testing.assert_allclose(QKV[:, :qw], Q[:, p["q_off"] * d:p["q_off"] * d + qw], atol=1e-13)
        np.testing.assert_allclose(QKV[:, qw:qw + kw], K[:, p["kv_off"] * d:p["kv_off"] * d + kw], atol=1e-13)
        np.testing.assert_allclose(QKV[:, qw + kw:], V[:, p["kv_off"] * d:p["kv_off"] * d + kw], atol=1e-13)
        # explicit loops for the row-parallel half
        ref = np.zeros((M, H))
        for m in range(M):
            for k in range(qw):
                for h in range(H):
                    ref[m, h] += C_i[m, k] * Wo_i[k, h]
        np.testing.assert_allclose(Zp, ref, atol=1e-12)


def test_attn_proj_bwd_finite_differences():
    # L = sum(QKV * dQKV) + sum(Zhat * dZ); the projections are bilinear so central differences are exact up to rounding.
    g = _rng(8)
    M, H, wqkv, wo = 3, 5, 4, 2
    X, Wqkv, C, Wo = (g.standard_normal((M, H)), g.standard_normal((H, wqkv)), g.standard_normal((M, wo)),
                      g.standard_normal((wo, H)))
    dZ, dQKV = g.standard_normal((M, H)), g.standard_normal((M, wqkv))

    def loss(Xv, Wv, Cv, Wov):
        qkv, z = O.attn_proj_shard_fwd(Xv, Wv, Cv, Wov)
        return float((qkv * dQKV).sum() + (z * dZ).sum())

    dC, dX, dWqkv, dWo = O.attn_proj_shard_bwd(dZ, dQKV, X, C, Wqkv, Wo)
    h = 1e-5
    for arr, grad, which in ((X, dX, 0), (Wqkv, dWqkv, 1), (C, dC, 2), (Wo, dWo, 3)):
        for idx in np.ndindex(arr.shape):
            args = [X.copy(), Wqkv.copy(), C.copy(), Wo.copy()]
            args[which][idx] += h
            up = loss(*args)
            args[which][idx] -= 2 * h
            dn = loss(*args)
            assert abs((up - dn) / (2 * h) - grad[idx]) < 1e-8 * max(1.0, abs(grad[idx]))
