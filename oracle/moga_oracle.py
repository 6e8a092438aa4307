"""CPU oracle for the Mixture-of-Groups Attention (MoGA) hot path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP kernels are checked against.  It is imported by the tests, by the smoke
check and by the benchmark's CPU-baseline leg, and by nothing else; it shares
no code with the GPU path and never calls it.

Everything is numpy in float64 unless a step says otherwise.  Each function
names the passage of the MoGA paper (arXiv 2510.18692) that it writes out:

  Eq. 1   vanilla self-attention          softmax(q K^T * scale) V
  Eq. 2   router scores                   r = Router(x), a single linear layer
  Eq. 3   group probabilities             p(i|x) = softmax(r)_i
  Eq. 4   top-1 assignment                g(x) = argmax_i p(i|x)
  Eq. 5   MoGA output                     p(g(x)|x) * SA(q, K_g, V_g)
  Alg. 1  router -> permute -> varlen attention -> repermute
  Eqs. 6-8 group balancing loss

Readings taken where the paper is silent (each is listed in the design notes):
  * the router is weight-only unless a bias is passed;
  * argmax is taken over the logits rounded to float32 (the precision the
    kernels decide in), lowest index on ties;
  * one group and one gate per token, shared by all heads;
  * attention is bidirectional, no dropout, scale passed in explicitly;
  * the permutation is stable: ascending token index within a group;
  * the gradient reaches the router only through the gate in Eq. 5; the
    assignment g is a constant of differentiation.

Pins (tests/test_oracle_*.py): M=1 equals plain full attention; the dense
masked definition on tiny inputs, itself pinned to pure-Python brute force;
closed forms (zero router weight, constant V, zero Q); permutation
invariants; group independence and token-order equivariance; log-sum-exp
against scipy; central finite differences for every gradient; the zero
column-sum of dW.  Parity unpinned: absolute output values on random inputs,
because the paper prints no token-level worked example.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "router_logits", "route", "permute_index", "permute", "softmax_attention",
    "group_attention", "group_attention_rows", "unpermute", "moga_forward",
    "dense_masked_moga", "softmax_attention_bwd", "softmax_attention_bwd_rows",
    "group_attention_bwd", "route_bwd", "moga_backward", "balance_loss",
    "balance_loss_bwd",
]


def _f64(a):
    return np.asarray(a, dtype=np.float64)


# --------------------------------------------------------------------------
# Router: Eqs. 2-4
# --------------------------------------------------------------------------
def router_logits(X, W, bias=None):
    """Eq. 2 with a single linear layer: r[i, j] = sum_c X[i, c] * W[j, c] (+ bias[j]).

    X [N, d], W [M, d]; float64 accumulation of the stored input values.
    """
    r = _f64(X) @ _f64(W).T
    if bias is not None:
        r = r + _f64(bias)[None, :]
    return r


def route(X, W, bias=None):
    """Eqs. 2-4 and the gate used by Eq. 5.

    Returns a dict with
      r64   [N, M] float64 logits,
      r32   [N, M] the same rounded to float32 (the precision argmax is taken in),
      group [N]    int32, argmax_j r32[i, j], lowest index on ties (Eq. 4; the
                   softmax of Eq. 3 is monotone so the argmax of p equals that of r),
      probs [N, M] float32 softmax(r) (Eq. 3), evaluated in float64,
      gate  [N]    float32 p(g(x)|x).
    """
    r64 = router_logits(X, W, bias)
    r32 = r64.astype(np.float32)
    group = np.argmax(r32, axis=1).astype(np.int32)  # first occurrence = lowest index
    top = np.take_along_axis(r64, group[:, None].astype(np.int64), axis=1)
    e = np.exp(r64 - top)
    denom = e.sum(axis=1, keepdims=True)
    probs = e / denom
    gate = 1.0 / denom[:, 0]
    return {
        "r64": r64,
        "r32": r32,
        "group": group,
        "probs": probs.astype(np.float32),
        "gate": gate.astype(np.float32),
    }


# --------------------------------------------------------------------------
# Permutation: Alg. 1 step 2
# --------------------------------------------------------------------------
def permute_index(group, M):
    """Histogram, offsets and the stable group-sorting permutation (Alg. 1 step 2).

    counts[g]     = number of tokens with group == g
    cu_seqlens    = exclusive prefix sum of counts, length M+1, cu[M] = N
    max_seqlen    = max(counts) (0 when N == 0)
    perm[j]       = token that lands in sorted slot j: group g occupies slots
                    cu[g]..cu[g+1], tokens in ascending index inside a group
    inv_perm[i]   = slot of token i
    All int32.
    """
    group = np.asarray(group)
    N = group.shape[0]
    if N and (group.min() < 0 or group.max() >= M):
        raise ValueError("group id out of range")
    counts = np.zeros(M, dtype=np.int32)
    for g in range(M):
        counts[g] = np.count_nonzero(group == g)
    cu = np.zeros(M + 1, dtype=np.int32)
    for g in range(M):
        cu[g + 1] = cu[g] + counts[g]
    perm = np.empty(N, dtype=np.int32)
    for g in range(M):
        members = np.nonzero(group == g)[0]  # ascending token index
        perm[cu[g]:cu[g + 1]] = members
    inv_perm = np.empty(N, dtype=np.int32)
    inv_perm[perm] = np.arange(N, dtype=np.int32)
    max_seqlen = np.int32(counts.max() if M > 0 and N > 0 else 0)
    return {"counts": counts, "cu_seqlens": cu, "max_seqlen": max_seqlen,
            "perm": perm, "inv_perm": inv_perm}


def permute(Q, K, V, group, M):
    """Alg. 1 step 2: gather Q, K, V ([N, H, D]) into group-contiguous order.

    Returns (Qh, Kh, Vh, index) with Qh[j] = Q[perm[j]] etc., still [N, H, D].
    """
    idx = permute_index(group, M)
    p = idx["perm"]
    return np.asarray(Q)[p], np.asarray(K)[p], np.asarray(V)[p], idx


# --------------------------------------------------------------------------
# Attention: Eq. 1 applied inside each group (Eq. 5, Alg. 1 step 3)
# --------------------------------------------------------------------------
def softmax_attention(q, K, V, scale):
    """Eq. 1 for one head: rows of q [n_q, D] attend to all of K, V [n_k, D].

    Returns (out [n_q, D], lse [n_q]) with lse = log sum_j exp(scale * q.k_j).
    """
    q, K, V = _f64(q), _f64(K), _f64(V)
    S = (q @ K.T) * scale
    m = S.max(axis=1, keepdims=True)
    P = np.exp(S - m)
    l = P.sum(axis=1, keepdims=True)
    out = (P / l) @ V
    lse = m[:, 0] + np.log(l[:, 0])
    return out, lse


def group_attention(Qh, Kh, Vh, cu_seqlens, scale):
    """Alg. 1 step 3: independent full softmax attention inside every group.

    Qh, Kh, Vh [N, H, D] in group-contiguous order; group g is rows cu[g]..cu[g+1].
    Returns (A [N, H, D] float64, lse [N, H] float64).  Empty groups do nothing.
    """
    Qh, Kh, Vh = _f64(Qh), _f64(Kh), _f64(Vh)
    N, H, D = Qh.shape
    A = np.zeros((N, H, D))
    lse = np.zeros((N, H))
    for g in range(len(cu_seqlens) - 1):
        s, e = int(cu_seqlens[g]), int(cu_seqlens[g + 1])
        if e == s:
            continue
        for h in range(H):
            A[s:e, h], lse[s:e, h] = softmax_attention(Qh[s:e, h], Kh[s:e, h], Vh[s:e, h], scale)
    return A, lse


def group_attention_rows(Qh, Kh, Vh, cu_seqlens, scale, g, h, rows):
    """The rows `rows` (offsets inside group g) of head h of `group_attention`, one by one.

    For sizes where the whole output is out of reach: each sampled query row is
    still attended against every key of its group, so the rows are exact.
    """
    s, e = int(cu_seqlens[g]), int(cu_seqlens[g + 1])
    rows = np.asarray(rows, dtype=np.int64)
    return softmax_attention(np.asarray(Qh)[s + rows, h], np.asarray(Kh)[s:e, h],
                             np.asarray(Vh)[s:e, h], scale)


def unpermute(A, perm, gate=None):
    """Alg. 1 step 4 with the gate of Eq. 5: O[perm[j]] = gate[perm[j]] * A[j]."""
    A = _f64(A)
    O = np.empty_like(A)
    O[perm] = A
    if gate is not None:
        O = O * _f64(gate)[:, None, None]
    return O


def moga_forward(X, W, Q, K, V, scale, bias=None, group_override=None):
    """Alg. 1 end to end with the gate of Eq. 5.

    X [N, d], W [M, d], Q/K/V [N, H, D].  `group_override` replaces the routed
    assignment (hand-assigned groups; the gate is still the router's p of that group).
    Returns a dict with every intermediate.
    """
    M = np.asarray(W).shape[0]
    rt = route(X, W, bias)
    group = rt["group"]
    gate = rt["gate"]
    if group_override is not None:
        group = np.asarray(group_override, dtype=np.int32)
        gate = np.take_along_axis(rt["probs"], group[:, None].astype(np.int64), axis=1)[:, 0]
    Qh, Kh, Vh, idx = permute(Q, K, V, group, M)
    A, lse = group_attention(Qh, Kh, Vh, idx["cu_seqlens"], scale)
    O = unpermute(A, idx["perm"], gate)
    out = dict(rt)
    out.update(idx)
    out.update({"group": group, "gate": gate, "Qh": Qh, "Kh": Kh, "Vh": Vh,
                "A": A, "lse": lse, "O": O})
    return out


def dense_masked_moga(X, W, Q, K, V, scale, bias=None):
    """Eq. 5 written as one dense masked attention (small N only).

    Token i attends to exactly the tokens j with g(j) == g(i); the result is
    multiplied by p(g(i)|x_i).  No permutation, no offsets: the definition
    against which the step-by-step path above is pinned.
    """
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    r = router_logits(X, W, bias)
    r32 = r.astype(np.float32)
    g = np.argmax(r32, axis=1)
    p = np.exp(r - r.max(axis=1, keepdims=True))
    p = p / p.sum(axis=1, keepdims=True)
    gate = p[np.arange(len(g)), g]
    mask = g[:, None] == g[None, :]
    N, H, D = Q.shape
    O = np.zeros((N, H, D))
    for h in range(H):
        S = (Q[:, h] @ K[:, h].T) * scale
        S = np.where(mask, S, -np.inf)
        S = S - S.max(axis=1, keepdims=True)
        P = np.exp(S)
        P = P / P.sum(axis=1, keepdims=True)
        O[:, h] = gate[:, None] * (P @ V[:, h])
    return O


# --------------------------------------------------------------------------
# Backward.  The paper states only that the router is trained end to end; the
# formulas below are the derivative of Eq. 5 with the assignment g held fixed.
# --------------------------------------------------------------------------
def softmax_attention_bwd(q, K, V, dA, scale):
    """Gradients of Eq. 1 for one head and one key set, with the explicit P matrix.

    q, dA [n, D]; K, V [n_k, D].  Returns (dq, dK, dV).
      P  = softmax(scale * q K^T)        dV = P^T dA
      dP = dA V^T                        dS = P * (dP - rowsum(dP * P))
      dq = scale * dS K                  dK = scale * dS^T q
    """
    q, K, V, dA = _f64(q), _f64(K), _f64(V), _f64(dA)
    S = (q @ K.T) * scale
    S = S - S.max(axis=1, keepdims=True)
    P = np.exp(S)
    P = P / P.sum(axis=1, keepdims=True)
    dV = P.T @ dA
    dP = dA @ V.T
    dS = P * (dP - (dP * P).sum(axis=1, keepdims=True))
    dq = scale * (dS @ K)
    dK = scale * (dS.T @ q)
    return dq, dK, dV


def softmax_attention_bwd_rows(q_rows, K, V, dA_rows, scale):
    """dq for a few query rows only (each row's gradient needs just its own P row)."""
    dq, _, _ = softmax_attention_bwd(q_rows, K, V, dA_rows, scale)
    return dq


def group_attention_bwd(Qh, Kh, Vh, dA, cu_seqlens, scale):
    """Backward of `group_attention`: per group, per head (all arrays [N, H, D])."""
    Qh, Kh, Vh, dA = _f64(Qh), _f64(Kh), _f64(Vh), _f64(dA)
    dQ, dK, dV = np.zeros_like(Qh), np.zeros_like(Kh), np.zeros_like(Vh)
    H = Qh.shape[1]
    for g in range(len(cu_seqlens) - 1):
        s, e = int(cu_seqlens[g]), int(cu_seqlens[g + 1])
        if e == s:
            continue
        for h in range(H):
            dQ[s:e, h], dK[s:e, h], dV[s:e, h] = softmax_attention_bwd(
                Qh[s:e, h], Kh[s:e, h], Vh[s:e, h], dA[s:e, h], scale)
    return dQ, dK, dV


def route_bwd(X, W, probs, group, gate, d_gate, want_dx=False):
    """Gradient of the gate p(g|x) (Eq. 3 at the chosen group) w.r.t. the router weight.

    dr[i, j] = d_gate[i] * gate[i] * ([j == g_i] - p[i, j])   (softmax Jacobian row g_i)
    dW       = dr^T X        [M, d]
    dX       = dr W          [N, d]  (only the router's contribution)
    """
    probs, gate, d_gate = _f64(probs), _f64(gate), _f64(d_gate)
    N, M = probs.shape
    onehot = np.zeros((N, M))
    onehot[np.arange(N), np.asarray(group, dtype=np.int64)] = 1.0
    dr = (d_gate * gate)[:, None] * (onehot - probs)
    dW = dr.T @ _f64(X)
    dX = dr @ _f64(W) if want_dx else None
    return dW, dX, dr


def moga_backward(fwd, X, W, dO, scale, want_dx=False):
    """Backward of `moga_forward` given its result dict `fwd` and dO [N, H, D].

    Returns dict(dQ, dK, dV [N, H, D] token order; dW [M, d]; d_gate [N]; dA, dQh, dKh, dVh
    in group-contiguous order; dr; dX when asked).
    """
    dO = _f64(dO)
    perm, gate = fwd["perm"], _f64(fwd["gate"])
    A = fwd["A"]                                   # ungated attention output, sorted order
    A_tok = np.empty_like(A)
    A_tok[perm] = A
    d_gate = (dO * A_tok).sum(axis=(1, 2))         # O_i = gate_i * A_i
    dA = (dO * gate[:, None, None])[perm]          # sorted order
    dQh, dKh, dVh = group_attention_bwd(fwd["Qh"], fwd["Kh"], fwd["Vh"], dA,
                                        fwd["cu_seqlens"], scale)
    dQ, dK, dV = np.empty_like(dQh), np.empty_like(dKh), np.empty_like(dVh)
    dQ[perm], dK[perm], dV[perm] = dQh, dKh, dVh
    # probabilities in float64 for the Jacobian (the stored float32 copy would lose digits)
    r = fwd["r64"]
    p = np.exp(r - r.max(axis=1, keepdims=True))
    p = p / p.sum(axis=1, keepdims=True)
    gate64 = p[np.arange(p.shape[0]), np.asarray(fwd["group"], dtype=np.int64)]
    dW, dX, dr = route_bwd(X, W, p, fwd["group"], gate64, d_gate, want_dx)
    return {"dQ": dQ, "dK": dK, "dV": dV, "dW": dW, "dX": dX, "d_gate": d_gate,
            "dA": dA, "dQh": dQh, "dKh": dKh, "dVh": dVh, "dr": dr}


# --------------------------------------------------------------------------
# Group balancing loss: Eqs. 6-8
# --------------------------------------------------------------------------
def balance_loss(group, gate, M, alpha):
    """Eqs. 6-8: L = alpha * M * sum_i F_i * P_i.

    F_i = (1/N) #{x : g(x) = i}                        (Eq. 7)
    P_i = (1/N) sum_{x : g(x) = i} p(g(x)|x)           (Eq. 8, read literally: the sum
          runs over the tokens assigned to i only)
    Returns (L, F [M], P [M]).
    """
    group = np.asarray(group, dtype=np.int64)
    gate = _f64(gate)
    N = group.shape[0]
    F = np.zeros(M)
    P = np.zeros(M)
    for i in range(M):
        sel = group == i
        F[i] = np.count_nonzero(sel) / N
        P[i] = gate[sel].sum() / N
    return alpha * M * float((F * P).sum()), F, P


def balance_loss_bwd(group, M, alpha):
    """dL/d gate[x] = alpha * M * F_{g(x)} / N  (F is piecewise constant in the weights)."""
    group = np.asarray(group, dtype=np.int64)
    N = group.shape[0]
    F = np.bincount(group, minlength=M).astype(np.float64) / N
    return alpha * M * F[group] / N
