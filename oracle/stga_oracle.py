"""CPU oracle for the static groups that accompany MoGA: spatial-temporal group attention
(STGA), per-frame attention and the mean of the three branches (Section 3.2, paragraph
"Spatial-Temporal Group Attention", and Fig. 2(a) of the MoGA paper, arXiv 2510.18692).

TEST INFRASTRUCTURE ONLY, like moga_oracle: plain numpy float64, imported by the tests and by
nothing in the product path; it shares no code with the HIP library.

What the paper states, restated:
  * the latent video is cut into fixed spatial windows, and frames are grouped along time;
    frames of different shots never share a temporal group;
  * a static group is (temporal group, spatial window); attention runs inside each group;
  * the keys and values of a group (not its queries) are extended by two latent frames taken
    from the adjacent shots;
  * a second static grouping puts all tokens of one latent frame in a group;
  * a token's final output is the mean of its outputs from the dynamic (MoGA) branch and the
    two static branches.

Readings taken where the paper gives no numbers or is ambiguous (listed in the design notes):
  * tokens are indexed frame-major, then row-major: i = (t * Hh + y) * Ww + x;
  * windows do not overlap; a window index is (y // wh, x // ww), ragged at the border;
  * inside a shot, temporal groups are consecutive runs of `tg` frames, the last one shorter;
  * "two latent frames from adjacent shots" = the last frame of the previous shot and the first
    frame of the next shot (`a_prev` = `a_next` = 1; other counts can be passed), restricted
    to the group's own spatial window; a shot at either end of the video has one neighbour;
  * within a group, own keys come first in ascending token order, then the added frames'
    tokens in ascending token order (the result does not depend on this order);
  * the static branches are not gated: the router probability of Eq. 5 multiplies only the
    dynamic branch.

Pins (tests/test_oracle_stga.py): the dense masked definition with the mask written directly
from (t, y, x, shot); one window + one temporal group + one shot = plain full attention;
partition invariants of the index lists; the attention-cost count against the closed form
sum over groups of n_q * n_k; finite differences for the backward; mean of three branches with
identical branches = that branch.  Parity unpinned: absolute values on random inputs (the paper
gives neither window sizes nor a worked example).
"""
from __future__ import annotations

import numpy as np

from . import moga_oracle as _mo

__all__ = [
    "token_coords", "stga_group_of_token", "frame_group_of_token", "stga_index", "frame_index",
    "varlen_attention", "varlen_attention_bwd", "dense_masked_attention", "visual_attention",
    "visual_attention_bwd", "attention_pairs",
]


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def token_coords(T, Hh, Ww):
    """(t, y, x) of every token, i = (t * Hh + y) * Ww + x."""
    i = np.arange(T * Hh * Ww)
    return i // (Hh * Ww), (i // Ww) % Hh, i % Ww


def _temporal_group_of_frame(shot_of_frame, tg):
    """Consecutive runs of `tg` frames inside each shot; returns the run id of every frame."""
    shot_of_frame = np.asarray(shot_of_frame, dtype=np.int64)
    out = np.zeros(len(shot_of_frame), dtype=np.int64)
    run = -1
    in_run = 0
    for t in range(len(shot_of_frame)):
        new_shot = t == 0 or shot_of_frame[t] != shot_of_frame[t - 1]
        if new_shot or in_run == tg:
            run += 1
            in_run = 0
        out[t] = run
        in_run += 1
    return out


def stga_group_of_token(T, Hh, Ww, wh, ww, tg, shot_of_frame):
    """Static group id of every token: temporal run * n_windows + window.  Returns (group [N], G)."""
    t, y, x = token_coords(T, Hh, Ww)
    nwy, nwx = -(-Hh // wh), -(-Ww // ww)
    run = _temporal_group_of_frame(shot_of_frame, tg)
    win = (y // wh) * nwx + (x // ww)
    G = int(run.max() + 1) * nwy * nwx
    return (run[t] * (nwy * nwx) + win).astype(np.int32), G


def frame_group_of_token(T, Hh, Ww):
    """Per-frame grouping: group = latent frame index."""
    t, _, _ = token_coords(T, Hh, Ww)
    return t.astype(np.int32), T


def stga_index(T, Hh, Ww, wh, ww, tg, shot_of_frame, a_prev=1, a_next=1):
    """Index lists of the STGA branch.

    Returns a dict of int32 arrays:
      q_index [N]    tokens sorted by (group, token): the queries of group g are
                     q_index[cu_q[g] : cu_q[g+1]]
      cu_q [G+1]
      kv_index [Nk]  keys/values of group g are kv_index[cu_k[g] : cu_k[g+1]]: the group's own
                     tokens (ascending), then the tokens of its spatial window in the last
                     a_prev frames of the previous shot and the first a_next frames of the next
                     shot (ascending)
      cu_k [G+1]
    """
    shot_of_frame = np.asarray(shot_of_frame, dtype=np.int64)
    group, G = stga_group_of_token(T, Hh, Ww, wh, ww, tg, shot_of_frame)
    t, y, x = token_coords(T, Hh, Ww)
    nwx = -(-Ww // ww)
    win = (y // wh) * nwx + (x // ww)
    run = _temporal_group_of_frame(shot_of_frame, tg)
    n_windows = (-(-Hh // wh)) * nwx
    shots = np.unique(shot_of_frame)
    frames_of_shot = {int(s): np.nonzero(shot_of_frame == s)[0] for s in shots}
    shot_list = [int(s) for s in shots]          # in order of appearance (non-decreasing ids)
    q_index, kv_index, cu_q, cu_k = [], [], [0], [0]
    for g in range(G):
        own = np.nonzero(group == g)[0]
        q_index.extend(own.tolist())
        kv = own.tolist()
        if len(own):
            r, w = divmod(g, n_windows)
            shot = int(shot_of_frame[np.nonzero(run == r)[0][0]])
            pos = shot_list.index(shot)
            extra_frames = []
            if pos > 0 and a_prev > 0:
                extra_frames.extend(frames_of_shot[shot_list[pos - 1]][-a_prev:].tolist())
            if pos + 1 < len(shot_list) and a_next > 0:
                extra_frames.extend(frames_of_shot[shot_list[pos + 1]][:a_next].tolist())
            for f in sorted(extra_frames):
                kv.extend(np.nonzero((t == f) & (win == w))[0].tolist())
        kv_index.extend(kv)
        cu_q.append(len(q_index))
        cu_k.append(len(kv_index))
    as32 = lambda a: np.asarray(a, dtype=np.int32)
    return {"q_index": as32(q_index), "cu_q": as32(cu_q), "kv_index": as32(kv_index), "cu_k": as32(cu_k),
            "n_groups": G}


def frame_index(T, Hh, Ww):
    """Index lists of the per-frame branch: group f = the tokens of latent frame f, keys = queries."""
    n = Hh * Ww
    idx = np.arange(T * n, dtype=np.int32)
    cu = (np.arange(T + 1) * n).astype(np.int32)
    return {"q_index": idx, "cu_q": cu, "kv_index": idx.copy(), "cu_k": cu.copy(), "n_groups": T}


def attention_pairs(cu_q, cu_k):
    """Number of (query, key) pairs the branch evaluates: sum over groups of n_q * n_k."""
    cu_q, cu_k = np.asarray(cu_q, dtype=np.int64), np.asarray(cu_k, dtype=np.int64)
    return int(((cu_q[1:] - cu_q[:-1]) * (cu_k[1:] - cu_k[:-1])).sum())


def varlen_attention(Q, K, V, q_index, cu_q, kv_index, cu_k, scale):
    """Eq. 1 inside every static group, queries and keys listed separately.

    Q, K, V [N, H, D] in token order.  Returns (A [N, H, D], lse [N, H]) in token order.  A token
    that is in no group's query list, or whose group has no keys, gets A = 0 and lse = -inf.
    """
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    N, H, D = Q.shape
    A = np.zeros((N, H, D))
    lse = np.full((N, H), -np.inf)
    for g in range(len(cu_q) - 1):
        qi = np.asarray(q_index[int(cu_q[g]):int(cu_q[g + 1])], dtype=np.int64)
        ki = np.asarray(kv_index[int(cu_k[g]):int(cu_k[g + 1])], dtype=np.int64)
        if len(qi) == 0 or len(ki) == 0:
            continue
        for h in range(H):
            A[qi, h], lse[qi, h] = _mo.softmax_attention(Q[qi, h], K[ki, h], V[ki, h], scale)
    return A, lse


def varlen_attention_bwd(Q, K, V, dA, q_index, cu_q, kv_index, cu_k, scale):
    """Backward of `varlen_attention` in token order; a token used as a key by several groups
    receives the sum of their contributions."""
    Q, K, V, dA = _f64(Q), _f64(K), _f64(V), _f64(dA)
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    H = Q.shape[1]
    for g in range(len(cu_q) - 1):
        qi = np.asarray(q_index[int(cu_q[g]):int(cu_q[g + 1])], dtype=np.int64)
        ki = np.asarray(kv_index[int(cu_k[g]):int(cu_k[g + 1])], dtype=np.int64)
        if len(qi) == 0 or len(ki) == 0:
            continue
        for h in range(H):
            dq, dk, dv = _mo.softmax_attention_bwd(Q[qi, h], K[ki, h], V[ki, h], dA[qi, h], scale)
            dQ[qi, h] += dq
            np.add.at(dK[:, h], ki, dk)
            np.add.at(dV[:, h], ki, dv)
    return dQ, dK, dV


def dense_masked_attention(Q, K, V, mask, scale):
    """Plain definition for tiny inputs: token i attends to every token j with mask[i, j] true.

    Rows with an empty mask give zero.  Three plain loops over heads and rows.
    """
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    N, H, D = Q.shape
    out = np.zeros((N, H, D))
    for h in range(H):
        for i in range(N):
            js = np.nonzero(mask[i])[0]
            if len(js) == 0:
                continue
            s = np.array([scale * float(np.dot(Q[i, h], K[j, h])) for j in js])
            p = np.exp(s - s.max())
            p /= p.sum()
            out[i, h] = sum(p[a] * V[j, h] for a, j in enumerate(js))
    return out


def visual_attention(X, W, Q, K, V, scale, grid, wh, ww, tg, shot_of_frame, a_prev=1, a_next=1):
    """Mean of the three branches: MoGA (Eq. 5, gated), STGA and per-frame attention.

    grid = (T, Hh, Ww) with T * Hh * Ww == N.  Returns a dict with the three branch outputs,
    their mean `O`, and the MoGA forward dict under "moga".
    """
    T, Hh, Ww = grid
    moga = _mo.moga_forward(X, W, Q, K, V, scale)
    si = stga_index(T, Hh, Ww, wh, ww, tg, shot_of_frame, a_prev, a_next)
    fi = frame_index(T, Hh, Ww)
    O_s, _ = varlen_attention(Q, K, V, si["q_index"], si["cu_q"], si["kv_index"], si["cu_k"], scale)
    O_f, _ = varlen_attention(Q, K, V, fi["q_index"], fi["cu_q"], fi["kv_index"], fi["cu_k"], scale)
    O = (moga["O"] + O_s + O_f) / 3.0
    return {"O": O, "O_moga": moga["O"], "O_stga": O_s, "O_frame": O_f, "moga": moga, "stga_index": si,
            "frame_index": fi}


def visual_attention_bwd(fwd, X, W, Q, K, V, dO, scale):
    """Backward of `visual_attention`: each branch receives dO / 3; gradients add up."""
    dO3 = _f64(dO) / 3.0
    b = _mo.moga_backward(fwd["moga"], X, W, dO3, scale)
    si, fi = fwd["stga_index"], fwd["frame_index"]
    dQs, dKs, dVs = varlen_attention_bwd(Q, K, V, dO3, si["q_index"], si["cu_q"], si["kv_index"], si["cu_k"], scale)
    dQf, dKf, dVf = varlen_attention_bwd(Q, K, V, dO3, fi["q_index"], fi["cu_q"], fi["kv_index"], fi["cu_k"], scale)
    return {"dQ": b["dQ"] + dQs + dQf, "dK": b["dK"] + dKs + dKf, "dV": b["dV"] + dVs + dVf, "dW": b["dW"]}
