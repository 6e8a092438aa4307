"""Pins of the STGA / per-frame / three-branch oracle (Section 3.2, "Spatial-Temporal Group
Attention") against things other than itself: the dense masked definition with the mask written
directly from token coordinates, plain full attention, partition invariants, a closed-form pair
count and finite differences."""
import numpy as np
import pytest

from oracle import moga_oracle as orc
from oracle import stga_oracle as sto


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def direct_mask(T, Hh, Ww, wh, ww, tg, shot, a_prev=1, a_next=1):
    """mask[i, j]: query token i may attend to key token j, written from the description alone:
    same window, and either the same temporal run of the same shot, or j lies in the last frame(s)
    of the shot before i's shot / the first frame(s) of the shot after it."""
    shot = np.asarray(shot)
    N = T * Hh * Ww
    first = {s: int(np.nonzero(shot == s)[0][0]) for s in np.unique(shot)}
    last = {s: int(np.nonzero(shot == s)[0][-1]) for s in np.unique(shot)}
    order = sorted(first, key=lambda s: first[s])
    mask = np.zeros((N, N), dtype=bool)
    for i in range(N):
        ti, yi, xi = i // (Hh * Ww), (i // Ww) % Hh, i % Ww
        si = shot[ti]
        pos = order.index(si)
        for j in range(N):
            tj, yj, xj = j // (Hh * Ww), (j // Ww) % Hh, j % Ww
            if (yi // wh, xi // ww) != (yj // wh, xj // ww):
                continue
            sj = shot[tj]
            if sj == si:
                mask[i, j] = (ti - first[si]) // tg == (tj - first[si]) // tg
            elif pos > 0 and sj == order[pos - 1]:
                mask[i, j] = tj > last[sj] - a_prev
            elif pos + 1 < len(order) and sj == order[pos + 1]:
                mask[i, j] = tj < first[sj] + a_next
    return mask


CASES = [
    # T, Hh, Ww, wh, ww, tg, shots
    (6, 4, 4, 2, 2, 2, [0, 0, 0, 1, 1, 1]),
    (7, 3, 5, 2, 3, 3, [0, 0, 1, 1, 1, 1, 2]),     # ragged windows, ragged runs, a one-frame shot
    (4, 2, 2, 2, 2, 4, [0, 0, 0, 0]),              # one shot: no added frames
    (5, 4, 2, 4, 1, 1, [3, 3, 5, 5, 9]),           # shot ids need not be 0..S-1
]


@pytest.mark.parametrize("T,Hh,Ww,wh,ww,tg,shot", CASES)
def test_index_lists_partition_the_tokens_and_match_the_direct_mask(T, Hh, Ww, wh, ww, tg, shot):
    N = T * Hh * Ww
    si = sto.stga_index(T, Hh, Ww, wh, ww, tg, shot)
    assert sorted(si["q_index"].tolist()) == list(range(N))          # every token is a query once
    assert si["cu_q"][0] == 0 and si["cu_q"][-1] == N and np.all(np.diff(si["cu_q"]) >= 0)
    assert si["cu_k"][-1] == len(si["kv_index"]) and np.all(np.diff(si["cu_k"]) >= np.diff(si["cu_q"]))
    group, G = sto.stga_group_of_token(T, Hh, Ww, wh, ww, tg, shot)
    assert G == si["n_groups"] == len(si["cu_q"]) - 1
    mask = direct_mask(T, Hh, Ww, wh, ww, tg, shot)
    built = np.zeros((N, N), dtype=bool)
    for g in range(G):
        q = si["q_index"][si["cu_q"][g]:si["cu_q"][g + 1]]
        k = si["kv_index"][si["cu_k"][g]:si["cu_k"][g + 1]]
        assert np.all(group[q] == g)
        assert len(set(k.tolist())) == len(k)                        # no key listed twice in a group
        built[np.ix_(q, k)] = True
    assert np.array_equal(built, mask)
    assert sto.attention_pairs(si["cu_q"], si["cu_k"]) == int(mask.sum())


@pytest.mark.parametrize("T,Hh,Ww,wh,ww,tg,shot", CASES[:2])
def test_varlen_attention_equals_the_dense_masked_definition(T, Hh, Ww, wh, ww, tg, shot):
    N, H, D = T * Hh * Ww, 2, 8
    Q, K, V = rnd((N, H, D), 1), rnd((N, H, D), 2), rnd((N, H, D), 3)
    si = sto.stga_index(T, Hh, Ww, wh, ww, tg, shot)
    A, lse = sto.varlen_attention(Q, K, V, si["q_index"], si["cu_q"], si["kv_index"], si["cu_k"], 0.3)
    ref = sto.dense_masked_attention(Q, K, V, direct_mask(T, Hh, Ww, wh, ww, tg, shot), 0.3)
    np.testing.assert_allclose(A, ref, rtol=1e-11, atol=1e-12)
    # lse against the definition for one token
    i, h = N // 2, 1
    js = np.nonzero(direct_mask(T, Hh, Ww, wh, ww, tg, shot)[i])[0]
    assert abs(lse[i, h] - np.log(np.exp(0.3 * K[js, h] @ Q[i, h]).sum())) < 1e-10


def test_per_frame_branch_is_block_diagonal_full_attention():
    T, Hh, Ww, H, D = 3, 2, 3, 2, 4
    N = T * Hh * Ww
    Q, K, V = rnd((N, H, D), 4), rnd((N, H, D), 5), rnd((N, H, D), 6)
    fi = sto.frame_index(T, Hh, Ww)
    A, _ = sto.varlen_attention(Q, K, V, fi["q_index"], fi["cu_q"], fi["kv_index"], fi["cu_k"], 0.5)
    n = Hh * Ww
    for f in range(T):
        for h in range(H):
            ref, _ = orc.softmax_attention(Q[f * n:(f + 1) * n, h], K[f * n:(f + 1) * n, h], V[f * n:(f + 1) * n, h], 0.5)
            np.testing.assert_allclose(A[f * n:(f + 1) * n, h], ref, rtol=1e-12, atol=1e-13)


def test_one_window_one_run_one_shot_is_plain_full_attention():
    T, Hh, Ww, H, D = 3, 2, 2, 1, 4
    N = T * Hh * Ww
    Q, K, V = rnd((N, H, D), 7), rnd((N, H, D), 8), rnd((N, H, D), 9)
    si = sto.stga_index(T, Hh, Ww, Hh, Ww, T, [0] * T)
    A, _ = sto.varlen_attention(Q, K, V, si["q_index"], si["cu_q"], si["kv_index"], si["cu_k"], 0.7)
    ref, _ = orc.softmax_attention(Q[:, 0], K[:, 0], V[:, 0], 0.7)
    np.testing.assert_allclose(A[:, 0], ref, rtol=1e-12, atol=1e-13)


def test_pair_count_closed_form_for_a_regular_video():
    """S shots of F frames, windows dividing the frame, runs dividing the shot: every group has
    tg * wh * ww queries; interior shots add 2 frames of keys, end shots add 1."""
    S, F, Hh, Ww, wh, ww, tg = 4, 6, 4, 6, 2, 3, 3
    shot = np.repeat(np.arange(S), F)
    si = sto.stga_index(S * F, Hh, Ww, wh, ww, tg, shot)
    nwin, runs = (Hh // wh) * (Ww // ww), F // tg
    nq, per_frame = tg * wh * ww, wh * ww
    expect = nwin * runs * (2 * nq * (nq + per_frame) + (S - 2) * nq * (nq + 2 * per_frame))
    assert sto.attention_pairs(si["cu_q"], si["cu_k"]) == expect


def test_backward_matches_finite_differences_including_shared_keys():
    T, Hh, Ww, wh, ww, tg, shot = 4, 2, 2, 1, 2, 1, [0, 0, 1, 1]
    N, H, D = T * Hh * Ww, 1, 3
    Q, K, V, R = rnd((N, H, D), 10), rnd((N, H, D), 11), rnd((N, H, D), 12), rnd((N, H, D), 13)
    si = sto.stga_index(T, Hh, Ww, wh, ww, tg, shot)
    # frame 1 (last of shot 0) is an added key frame for both runs of shot 1: multiplicity > 1
    counts = np.bincount(si["kv_index"], minlength=N)
    assert counts.max() >= 3
    f = lambda q, k, v: (sto.varlen_attention(q, k, v, si["q_index"], si["cu_q"], si["kv_index"], si["cu_k"], 0.4)[0] * R).sum()
    dQ, dK, dV = sto.varlen_attention_bwd(Q, K, V, R, si["q_index"], si["cu_q"], si["kv_index"], si["cu_k"], 0.4)
    eps = 1e-6
    for name, X, g in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for idx in [(0, 0, 0), (5, 0, 2), (N - 1, 0, 1), (4, 0, 0)]:
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += eps
            Xm[idx] -= eps
            args_p = [Xp if n == name else Y for n, Y in (("Q", Q), ("K", K), ("V", V))]
            args_m = [Xm if n == name else Y for n, Y in (("Q", Q), ("K", K), ("V", V))]
            fd = (f(*args_p) - f(*args_m)) / (2 * eps)
            assert abs(fd - g[idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, g[idx])


def test_three_branch_mean_and_its_gradient():
    T, Hh, Ww, H, D, d, M = 4, 2, 3, 2, 4, 6, 3
    N = T * Hh * Ww
    X, W = rnd((N, d), 20), rnd((M, d), 21) * 0.7
    Q, K, V, R = rnd((N, H, D), 22), rnd((N, H, D), 23), rnd((N, H, D), 24), rnd((N, H, D), 25)
    shot = [0, 0, 1, 1]
    fw = sto.visual_attention(X, W, Q, K, V, 0.5, (T, Hh, Ww), 2, 3, 2, shot)
    np.testing.assert_allclose(fw["O"], (fw["O_moga"] + fw["O_stga"] + fw["O_frame"]) / 3, rtol=0, atol=1e-15)
    np.testing.assert_allclose(fw["O_moga"], orc.dense_masked_moga(X, W, Q, K, V, 0.5), rtol=3e-7, atol=1e-9)  # gate is stored as float32
    bw = sto.visual_attention_bwd(fw, X, W, Q, K, V, R, 0.5)
    # the forward stores the gate as float32, too coarse for a difference quotient in W: the dynamic
    # branch of the loss is evaluated with the dense float64 definition instead
    def loss(q, k, v, w):
        f = sto.visual_attention(X, w, q, k, v, 0.5, (T, Hh, Ww), 2, 3, 2, shot)
        return ((orc.dense_masked_moga(X, w, q, k, v, 0.5) + f["O_stga"] + f["O_frame"]) / 3 * R).sum()
    eps = 1e-6
    for name, idx in (("Q", (3, 1, 2)), ("K", (7, 0, 0)), ("V", (N - 1, 1, 3)), ("W", (1, 4))):
        base = {"Q": Q, "K": K, "V": V, "W": W}
        p, m = {k: v.copy() for k, v in base.items()}, {k: v.copy() for k, v in base.items()}
        p[name][idx] += eps
        m[name][idx] -= eps
        fd = (loss(p["Q"], p["K"], p["V"], p["W"]) - loss(m["Q"], m["K"], m["V"], m["W"])) / (2 * eps)
        got = bw["d" + name][idx]
        assert abs(fd - got) <= 2e-6 * max(1.0, abs(fd)), (name, fd, got)
