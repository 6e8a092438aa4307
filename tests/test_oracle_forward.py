"""Pins for the forward half of the CPU oracle (no GPU).

Each test checks the oracle against something other than itself: a pure-Python
brute force of Eqs. 1-5, a closed form, an invariant, or a library routine.
"""
import math

import numpy as np
import pytest
from scipy.special import logsumexp

from oracle import moga_oracle as orc


def rand_case(seed, N=48, H=2, D=8, d=16, M=4, wscale=1.0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((N, d))
    W = rng.standard_normal((M, d)) * wscale / math.sqrt(d)
    Q = rng.standard_normal((N, H, D))
    K = rng.standard_normal((N, H, D))
    V = rng.standard_normal((N, H, D))
    return X, W, Q, K, V


# ---- pure-Python brute force of Eqs. 1-5 (lists and math.exp only) ----------
def brute_force_moga(X, W, Q, K, V, scale):
    N, H, D = Q.shape
    M, d = W.shape
    group, gate = [], []
    for i in range(N):
        r = [sum(float(X[i][c]) * float(W[j][c]) for c in range(d)) for j in range(M)]
        r32 = [float(np.float32(v)) for v in r]
        g = max(range(M), key=lambda j: (r32[j], -j))       # largest logit, lowest index on ties
        z = sum(math.exp(v - r[g]) for v in r)
        group.append(g)
        gate.append(1.0 / z)
    O = np.zeros((N, H, D))
    for i in range(N):
        members = [j for j in range(N) if group[j] == group[i]]
        for h in range(H):
            s = [scale * sum(float(Q[i][h][c]) * float(K[j][h][c]) for c in range(D)) for j in members]
            mx = max(s)
            e = [math.exp(v - mx) for v in s]
            z = sum(e)
            for c in range(D):
                O[i][h][c] = gate[i] * sum(e[t] / z * float(V[members[t]][h][c]) for t in range(len(members)))
    return np.array(group), np.array(gate), O


def test_dense_definition_matches_pure_python_brute_force():
    X, W, Q, K, V = rand_case(0, N=20, H=2, D=4, d=6, M=3)
    g, gate, O = brute_force_moga(X, W, Q, K, V, 0.5)
    np.testing.assert_allclose(orc.dense_masked_moga(X, W, Q, K, V, 0.5), O, rtol=1e-12, atol=1e-13)
    f = orc.moga_forward(X, W, Q, K, V, 0.5)
    assert np.array_equal(f["group"], g)
    np.testing.assert_allclose(f["gate"], gate, rtol=1e-6)
    np.testing.assert_allclose(f["O"], O, rtol=2e-6, atol=1e-7)  # gate is stored as float32


@pytest.mark.parametrize("M", [1, 2, 5, 8])
def test_stepwise_path_equals_dense_masked_definition(M):
    X, W, Q, K, V = rand_case(10 + M, N=200, H=3, D=16, d=32, M=M, wscale=2.0)
    f = orc.moga_forward(X, W, Q, K, V, 0.25)
    ref = orc.dense_masked_moga(X, W, Q, K, V, 0.25)
    np.testing.assert_allclose(f["O"], ref, rtol=2e-6, atol=1e-7)


def test_single_group_is_plain_full_attention():
    """M = 1: softmax over one logit is 1, so Eq. 5 reduces to Eq. 1 (Table 4, row M = 1)."""
    X, W, Q, K, V = rand_case(3, N=64, H=2, D=8, d=16, M=1)
    f = orc.moga_forward(X, W, Q, K, V, 0.3)
    assert np.all(f["group"] == 0) and np.all(f["gate"] == 1.0)
    # independent dense attention, written with an explicit loop over rows
    N, H, D = Q.shape
    ref = np.zeros_like(Q)
    for h in range(H):
        for i in range(N):
            s = 0.3 * (K[:, h] @ Q[i, h])
            w = np.exp(s - logsumexp(s))
            ref[i, h] = w @ V[:, h]
    np.testing.assert_allclose(f["O"], ref, rtol=1e-11, atol=1e-12)


def test_zero_router_weight_ties_go_to_group_zero_and_gate_is_one_over_M():
    X, W, Q, K, V = rand_case(4, M=5)
    W = np.zeros_like(W)
    f = orc.moga_forward(X, W, Q, K, V, 0.3)
    assert np.all(f["group"] == 0)
    np.testing.assert_allclose(f["gate"], 1.0 / 5, rtol=1e-7)
    full = orc.moga_forward(X, W[:1], Q, K, V, 0.3)["O"]  # M = 1 is full attention
    np.testing.assert_allclose(f["O"], full / 5, rtol=1e-6)


def test_large_router_scale_drives_gate_to_one():
    X, W, Q, K, V = rand_case(5, M=4)
    f = orc.route(X, W * 1e4, None)
    assert np.all(f["gate"] > 1.0 - 1e-6)


def test_constant_value_rows_give_gate_times_value():
    """V_j = v for all j: any softmax average returns v, so O_i = gate_i * v for every head."""
    X, W, Q, K, V = rand_case(6, M=4)
    v = np.random.default_rng(1).standard_normal((V.shape[1], V.shape[2]))
    V = np.broadcast_to(v, V.shape).copy()
    f = orc.moga_forward(X, W, Q, K, V, 0.3)
    np.testing.assert_allclose(f["O"], f["gate"].astype(np.float64)[:, None, None] * v[None],
                               rtol=1e-12)


def test_zero_queries_give_group_mean_of_values():
    X, W, Q, K, V = rand_case(7, M=4)
    f = orc.moga_forward(X, W, np.zeros_like(Q), K, V, 0.3)
    for i in range(Q.shape[0]):
        members = f["group"] == f["group"][i]
        np.testing.assert_allclose(f["O"][i], f["gate"][i].astype(np.float64) * V[members].mean(axis=0),
                                   rtol=1e-11, atol=1e-13)


def test_bias_is_added_to_logits():
    X, W, Q, K, V = rand_case(8, M=4)
    b = np.array([0.0, 50.0, 0.0, 0.0])
    f = orc.route(X, W, b)
    assert np.all(f["group"] == 1)
    np.testing.assert_allclose(f["r64"], X @ W.T + b, rtol=1e-13)


def test_logits_are_x_times_w_transposed_not_the_reverse():
    X = np.array([[1.0, 2.0, 3.0]])
    W = np.array([[1.0, 0.0, 0.0], [0.0, 0.0, 2.0]])
    r = orc.router_logits(X, W)
    assert r.tolist() == [[1.0, 6.0]]
    f = orc.route(X, W)
    assert f["group"].tolist() == [1]
    p = math.exp(6) / (math.exp(1) + math.exp(6))
    assert abs(float(f["gate"][0]) - p) < 1e-7
    np.testing.assert_allclose(f["probs"][0], [1 - p, p], rtol=1e-6)


def test_probs_rows_sum_to_one_and_gate_is_the_row_max():
    X, W, *_ = rand_case(9, N=300, M=7, wscale=3.0)
    f = orc.route(X, W)
    np.testing.assert_allclose(f["probs"].sum(1), 1.0, rtol=1e-6)
    np.testing.assert_allclose(f["gate"], f["probs"].max(1), rtol=1e-6)
    assert np.array_equal(f["group"], f["probs"].astype(np.float64).argmax(1))


# ---- permutation ------------------------------------------------------------
def python_counting_sort(group, M):
    counts = [0] * M
    for g in group:
        counts[g] += 1
    cu = [0]
    for c in counts:
        cu.append(cu[-1] + c)
    nxt = cu[:-1].copy()
    perm = [0] * len(group)
    for i, g in enumerate(group):
        perm[nxt[g]] = i
        nxt[g] += 1
    return counts, cu, perm


@pytest.mark.parametrize("N,M", [(0, 3), (1, 1), (7, 4), (1000, 8), (5000, 32), (513, 256)])
def test_permutation_invariants_and_stable_sort(N, M):
    rng = np.random.default_rng(N + M)
    group = rng.integers(0, M, size=N).astype(np.int32)
    if N > 10:
        group[group == 1] = 0           # leave group 1 empty
    idx = orc.permute_index(group, M)
    counts, cu, perm = python_counting_sort(group.tolist(), M)
    assert idx["counts"].tolist() == counts
    assert idx["cu_seqlens"].tolist() == cu
    assert idx["perm"].tolist() == perm
    assert idx["perm"].tolist() == np.argsort(group, kind="stable").tolist()
    assert int(idx["max_seqlen"]) == (max(counts) if N else 0)
    assert idx["counts"].sum() == N and idx["cu_seqlens"][0] == 0 and idx["cu_seqlens"][-1] == N
    assert sorted(idx["perm"].tolist()) == list(range(N))
    assert np.array_equal(idx["inv_perm"][idx["perm"]], np.arange(N))
    keys = list(zip(group[idx["perm"]].tolist(), idx["perm"].tolist()))
    assert all(a < b for a, b in zip(keys, keys[1:]))
    for a in ("counts", "cu_seqlens", "perm", "inv_perm"):
        assert idx[a].dtype == np.int32


def test_permute_rejects_out_of_range_group():
    with pytest.raises(ValueError):
        orc.permute_index(np.array([0, 3]), 3)


# ---- attention inside groups ------------------------------------------------
def test_lse_matches_scipy_logsumexp_and_rows_of_p_sum_to_one():
    rng = np.random.default_rng(11)
    q, K, V = rng.standard_normal((5, 8)), rng.standard_normal((9, 8)), rng.standard_normal((9, 8))
    out, lse = orc.softmax_attention(q, K, V, 0.7)
    S = 0.7 * q @ K.T
    np.testing.assert_allclose(lse, logsumexp(S, axis=1), rtol=1e-13)
    P = np.exp(S - lse[:, None])
    np.testing.assert_allclose(P.sum(1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(out, P @ V, rtol=1e-12)


def test_attention_uses_keys_as_rows_of_the_score_matrix_columns():
    """Asymmetric check: one query identical to key 2 with a huge scale picks value 2."""
    K = np.eye(4)
    V = np.arange(16.0).reshape(4, 4)
    out, _ = orc.softmax_attention(K[2:3] * 100, K, V, 1.0)
    np.testing.assert_allclose(out[0], V[2], atol=1e-12)


def test_hand_assigned_contiguous_groups_are_block_diagonal_attention():
    X, W, Q, K, V = rand_case(12, N=60, M=3)
    go = np.repeat(np.arange(3), 20).astype(np.int32)
    f = orc.moga_forward(X, W, Q, K, V, 0.3, group_override=go)
    assert np.array_equal(f["perm"], np.arange(60))
    for b in range(3):
        sl = slice(20 * b, 20 * b + 20)
        for h in range(Q.shape[1]):
            ref, _ = orc.softmax_attention(Q[sl, h], K[sl, h], V[sl, h], 0.3)
            np.testing.assert_allclose(f["A"][sl, h], ref, rtol=1e-13)
    np.testing.assert_allclose(f["O"], f["gate"].astype(np.float64)[:, None, None] * f["A"], rtol=1e-13)


def test_groups_are_independent():
    """Perturbing Q/K/V of one group's tokens leaves every other group's output bit-identical."""
    X, W, Q, K, V = rand_case(13, N=120, M=4, wscale=2.0)
    f0 = orc.moga_forward(X, W, Q, K, V, 0.3)
    a = int(f0["group"][0])
    sel = f0["group"] == a
    Q2, K2, V2 = Q.copy(), K.copy(), V.copy()
    Q2[sel] += 1.0
    K2[sel] *= -2.0
    V2[sel] += 3.0
    f1 = orc.moga_forward(X, W, Q2, K2, V2, 0.3)
    assert np.array_equal(f0["O"][~sel], f1["O"][~sel])
    assert not np.allclose(f0["O"][sel], f1["O"][sel])


def test_token_order_equivariance():
    """Permuting tokens (X, Q, K, V together) permutes O the same way."""
    X, W, Q, K, V = rand_case(14, N=90, M=4, wscale=2.0)
    s = np.random.default_rng(2).permutation(90)
    f0 = orc.moga_forward(X, W, Q, K, V, 0.3)
    f1 = orc.moga_forward(X[s], W, Q[s], K[s], V[s], 0.3)
    np.testing.assert_allclose(f1["O"], f0["O"][s], rtol=1e-11, atol=1e-14)
    assert np.array_equal(f1["group"], f0["group"][s])


def test_group_of_one_returns_its_value_and_empty_groups_are_skipped():
    X, W, Q, K, V = rand_case(15, N=10, M=4)
    go = np.array([2, 0, 0, 0, 0, 0, 0, 0, 0, 0], dtype=np.int32)   # groups 1, 3 empty; group 2 single
    f = orc.moga_forward(X, W, Q, K, V, 0.3, group_override=go)
    assert f["counts"].tolist() == [9, 0, 1, 0]
    np.testing.assert_allclose(f["A"][9], V[0], rtol=1e-14)
    assert np.all(np.isfinite(f["O"]))


def test_rows_variant_equals_full_group_attention():
    X, W, Q, K, V = rand_case(16, N=150, M=3, wscale=2.0)
    f = orc.moga_forward(X, W, Q, K, V, 0.3)
    g = 1
    n = int(f["counts"][g])
    rows = np.array([0, n // 2, n - 1])
    out, lse = orc.group_attention_rows(f["Qh"], f["Kh"], f["Vh"], f["cu_seqlens"], 0.3, g, 1, rows)
    s = int(f["cu_seqlens"][g])
    np.testing.assert_allclose(out, f["A"][s + rows, 1], rtol=1e-13)
    np.testing.assert_allclose(lse, f["lse"][s + rows, 1], rtol=1e-13)


def test_gate_is_shared_by_all_heads():
    X, W, Q, K, V = rand_case(17, N=40, H=3, M=4)
    f = orc.moga_forward(X, W, Q, K, V, 0.3)
    A_tok = np.empty_like(f["A"])
    A_tok[f["perm"]] = f["A"]
    ratio = f["O"] / A_tok
    np.testing.assert_allclose(ratio, np.broadcast_to(f["gate"].astype(np.float64)[:, None, None], ratio.shape),
                               rtol=1e-10)


# ---- group balancing loss (Eqs. 6-8) -----------------------------------------
def test_balance_loss_uniform_assignment_with_uniform_probability_equals_alpha_over_m_times_m():
    """Uniform groups, gate = 1/M: F_i = 1/M, P_i = 1/M^2, L = alpha*M*M*(1/M^3) = alpha/M."""
    M, N, alpha = 4, 400, 0.1
    group = np.arange(N) % M
    gate = np.full(N, 1.0 / M)
    L, F, P = orc.balance_loss(group, gate, M, alpha)
    np.testing.assert_allclose(F, 1.0 / M)
    np.testing.assert_allclose(P, 1.0 / M ** 2)
    assert abs(L - alpha / M) < 1e-15


def test_balance_loss_confident_uniform_router_equals_alpha_and_collapse_is_worse():
    """gate -> 1: uniform assignment gives L = alpha (metric L/alpha = 1, App. B); collapse gives alpha*M."""
    M, N, alpha = 5, 500, 0.1
    L_uniform, _, _ = orc.balance_loss(np.arange(N) % M, np.ones(N), M, alpha)
    L_collapse, _, _ = orc.balance_loss(np.zeros(N, dtype=int), np.ones(N), M, alpha)
    assert abs(L_uniform - alpha) < 1e-15
    assert abs(L_collapse - alpha * M) < 1e-15


def test_balance_loss_gradient_matches_finite_difference_in_gate():
    rng = np.random.default_rng(3)
    M, N, alpha = 3, 30, 0.1
    group = rng.integers(0, M, N)
    gate = rng.uniform(0.4, 1.0, N)
    g = orc.balance_loss_bwd(group, M, alpha)
    for i in (0, 7, 29):
        e = np.zeros(N)
        e[i] = 1e-6
        fd = (orc.balance_loss(group, gate + e, M, alpha)[0] - orc.balance_loss(group, gate - e, M, alpha)[0]) / 2e-6
        assert abs(fd - g[i]) < 1e-9
