"""Pins for the backward half of the CPU oracle (no GPU).

The paper gives no backward formulas, so every gradient is pinned to central
finite differences of the forward oracle in float64, plus closed-form cases.
"""
import math

import numpy as np
import pytest

from oracle import moga_oracle as orc


def rand_case(seed, N=24, H=2, D=4, d=6, M=3, wscale=3.0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((N, d))
    W = rng.standard_normal((M, d)) * wscale / math.sqrt(d)
    Q = rng.standard_normal((N, H, D))
    K = rng.standard_normal((N, H, D))
    V = rng.standard_normal((N, H, D))
    R = rng.standard_normal((N, H, D))        # dO: loss = sum(O * R)
    return X, W, Q, K, V, R


def loss(X, W, Q, K, V, R, scale, group):
    # assignment held fixed (as the derivation does); gate recomputed from W
    f = orc.moga_forward(X, W, Q, K, V, scale, group_override=group)
    r = f["r64"]
    p = np.exp(r - r.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    gate = p[np.arange(len(group)), group]     # float64 gate (the stored one is float32)
    A_tok = np.empty_like(f["A"])
    A_tok[f["perm"]] = f["A"]
    return float((gate[:, None, None] * A_tok * R).sum())


def fd_grad(fun, arr, eps=1e-6, picks=None):
    g = np.zeros_like(arr)
    it = picks if picks is not None else list(np.ndindex(arr.shape))
    for idx in it:
        old = arr[idx]
        arr[idx] = old + eps
        fp = fun()
        arr[idx] = old - eps
        fm = fun()
        arr[idx] = old
        g[idx] = (fp - fm) / (2 * eps)
    return g


@pytest.mark.parametrize("seed,M", [(0, 3), (1, 1), (2, 5)])
def test_all_gradients_match_central_finite_differences(seed, M):
    X, W, Q, K, V, R = rand_case(seed, M=M)
    scale = 0.6
    f = orc.moga_forward(X, W, Q, K, V, scale)
    group = f["group"].astype(np.int64)
    b = orc.moga_backward(f, X, W, R, scale, want_dx=True)
    fun = lambda: loss(X, W, Q, K, V, R, scale, group)
    for name, arr in (("dQ", Q), ("dK", K), ("dV", V), ("dW", W), ("dX", X)):
        num = fd_grad(fun, arr)
        if name == "dX":
            pass  # only the router's contribution exists: Q, K, V are independent inputs here
        np.testing.assert_allclose(b[name], num, rtol=2e-6, atol=2e-8, err_msg=name)


def test_d_gate_matches_finite_difference_of_a_free_gate():
    X, W, Q, K, V, R = rand_case(3)
    f = orc.moga_forward(X, W, Q, K, V, 0.6)
    b = orc.moga_backward(f, X, W, R, 0.6)
    A_tok = np.empty_like(f["A"])
    A_tok[f["perm"]] = f["A"]
    # O_i = gate_i * A_i is linear in gate_i: the derivative is exactly sum(R_i * A_i)
    np.testing.assert_allclose(b["d_gate"], (R * A_tok).sum(axis=(1, 2)), rtol=1e-13)


def test_single_group_gives_textbook_attention_gradients_and_zero_router_gradient():
    X, W, Q, K, V, R = rand_case(4, M=1)
    f = orc.moga_forward(X, W, Q, K, V, 0.6)
    b = orc.moga_backward(f, X, W, R, 0.6)
    assert np.all(b["dW"] == 0.0)
    # textbook full-attention gradient for head 0 by finite differences on plain Eq. 1
    def full(h=0):
        S = 0.6 * Q[:, h] @ K[:, h].T
        P = np.exp(S - S.max(1, keepdims=True))
        P /= P.sum(1, keepdims=True)
        return float(((P @ V[:, h]) * R[:, h]).sum())
    picks = [(i, 0, c) for i in (0, 5, 23) for c in range(4)]
    for name, arr in (("dQ", Q), ("dK", K), ("dV", V)):
        num = fd_grad(full, arr, picks=picks)
        for idx in picks:
            assert abs(b[name][idx] - num[idx]) < 2e-7, (name, idx)


@pytest.mark.parametrize("M", [2, 4, 7])
def test_rows_of_dr_and_columns_of_dw_sum_to_zero(M):
    """Softmax Jacobian: sum_j dr[i, j] = 0 for every token, hence sum_j dW[j, :] = 0."""
    X, W, Q, K, V, R = rand_case(5 + M, N=60, M=M)
    f = orc.moga_forward(X, W, Q, K, V, 0.6)
    b = orc.moga_backward(f, X, W, R, 0.6)
    np.testing.assert_allclose(b["dr"].sum(1), 0.0, atol=1e-13)
    np.testing.assert_allclose(b["dW"].sum(0), 0.0, atol=1e-11)
    assert np.abs(b["dW"]).max() > 1e-3


def test_constant_value_rows_give_closed_form_d_gate_and_zero_attention_gradients():
    """V_j = v: A_i = v regardless of Q, K, so d_gate_i = sum(dO_i * v) and dQ = dK = 0."""
    X, W, Q, K, V, R = rand_case(6)
    v = np.random.default_rng(9).standard_normal(V.shape[1:])
    V = np.broadcast_to(v, V.shape).copy()
    f = orc.moga_forward(X, W, Q, K, V, 0.6)
    b = orc.moga_backward(f, X, W, R, 0.6)
    np.testing.assert_allclose(b["d_gate"], (R * v[None]).sum(axis=(1, 2)), rtol=1e-12)
    np.testing.assert_allclose(b["dQ"], 0.0, atol=1e-13)
    np.testing.assert_allclose(b["dK"], 0.0, atol=1e-13)


def test_dv_sums_to_gated_upstream_gradient_per_group():
    """Rows of P sum to one, so sum_j dV_j over a group = sum_i gate_i dO_i over that group."""
    X, W, Q, K, V, R = rand_case(7, N=50)
    f = orc.moga_forward(X, W, Q, K, V, 0.6)
    b = orc.moga_backward(f, X, W, R, 0.6)
    for g in range(W.shape[0]):
        sel = f["group"] == g
        np.testing.assert_allclose(b["dV"][sel].sum(0),
                                   (f["gate"].astype(np.float64)[sel, None, None] * R[sel]).sum(0),
                                   rtol=1e-11, atol=1e-13)


def test_rows_variant_of_dq_equals_the_full_backward():
    rng = np.random.default_rng(8)
    q, K, V, dA = (rng.standard_normal((12, 8)) for _ in range(4))
    dq, dK, dV = orc.softmax_attention_bwd(q, K, V, dA, 0.4)
    rows = np.array([0, 5, 11])
    np.testing.assert_allclose(orc.softmax_attention_bwd_rows(q[rows], K, V, dA[rows], 0.4), dq[rows],
                               rtol=1e-13)


def test_route_bwd_matches_finite_difference_of_the_gate_alone():
    rng = np.random.default_rng(10)
    N, d, M = 9, 5, 4
    X = rng.standard_normal((N, d))
    W = rng.standard_normal((M, d))
    c = rng.standard_normal(N)                   # loss = sum_i c_i * gate_i(W)
    rt = orc.route(X, W)
    group = rt["group"].astype(np.int64)

    def gate_of(Wm):
        r = X @ Wm.T
        p = np.exp(r - r.max(1, keepdims=True))
        p /= p.sum(1, keepdims=True)
        return p, p[np.arange(N), group]

    p, gate = gate_of(W)
    dW, dX, _ = orc.route_bwd(X, W, p, group, gate, c, want_dx=True)
    num = fd_grad(lambda: float((c * gate_of(W)[1]).sum()), W)
    np.testing.assert_allclose(dW, num, rtol=1e-6, atol=1e-9)
    Xc = X.copy()

    def loss_x():
        r = Xc @ W.T
        pp = np.exp(r - r.max(1, keepdims=True))
        pp /= pp.sum(1, keepdims=True)
        return float((c * pp[np.arange(N), group]).sum())
    np.testing.assert_allclose(dX, fd_grad(loss_x, Xc), rtol=1e-6, atol=1e-9)
