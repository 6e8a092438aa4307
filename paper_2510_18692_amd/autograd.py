"""torch.autograd wrappers around the C-ABI calls (argument marshalling only).

    o, lb = moga_attention(x, w, q, k, v, scale, balance_alpha=0.1)

`o` is the output of Alg. 1 with the gate of Eq. 5, `lb` the group balancing loss of Eqs. 6-8 (or
None).  Gradients flow to q, k, v and to the router weight w (through the gate, and through the
balancing loss when it is used); the assignment itself is a constant of differentiation.  No
gradient is returned for the router input x unless `grad_x=True` (the optional dX of the router
backward).  Everything runs in the HIP library; there is no fallback.
"""
from __future__ import annotations

import torch

from . import binding as mg


class _MogaAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, w, q, k, v, scale, balance_alpha, grad_x):
        fwd = mg.moga_forward(x, w, q, k, v, scale, want_probs=True)
        M = w.shape[0]
        ctx.scale, ctx.alpha, ctx.grad_x, ctx.M = scale, balance_alpha, grad_x, M
        ctx.fwd = fwd
        ctx.save_for_backward(x, w)
        if balance_alpha is not None:
            loss, frac, _ = mg.moga_balance_loss(fwd["group"], fwd["gate"], M, balance_alpha)
            ctx.frac = frac
            ctx.mark_non_differentiable(fwd["group"])
            return fwd["o"], loss[0], fwd["group"]
        ctx.mark_non_differentiable(fwd["group"])
        return fwd["o"], x.new_zeros((), dtype=torch.float32), fwd["group"]

    @staticmethod
    def backward(ctx, d_o, d_loss, _d_group):
        x, w = ctx.saved_tensors
        fwd = ctx.fwd
        d_o = d_o.contiguous()
        d_oh, d_gate = mg.moga_unpermute_bwd(d_o, fwd["oh"], fwd["perm"], fwd["gate"])
        d_qh, d_kh, d_vh = mg.moga_group_attn_bwd(d_oh, fwd["qh"], fwd["kh"], fwd["vh"], fwd["oh"], fwd["lse"],
                                                  fwd["cu_seqlens"], ctx.scale)
        d_q, d_k, d_v = mg.moga_permute_bwd(d_qh, d_kh, d_vh, fwd["perm"])
        if ctx.alpha is not None and d_loss is not None:
            mg.moga_balance_loss_bwd(fwd["group"], ctx.frac, ctx.alpha, d_loss=d_loss, d_gate=d_gate)
        d_w, d_x = mg.moga_route_bwd(x, w, fwd["probs"], fwd["group"], fwd["gate"], d_gate, want_dx=ctx.grad_x)
        if d_x is not None:
            d_x = d_x.to(x.dtype)
        ctx.fwd = None
        return d_x, d_w, d_q, d_k, d_v, None, None, None


def moga_attention(x, w, q, k, v, softmax_scale, balance_alpha=None, grad_x=False):
    """x [N, d_model], w [M, d_model] fp32, q/k/v [N, H, D] -> (o [N, H, D], balancing loss or None, group [N])."""
    o, loss, group = _MogaAttention.apply(x, w, q, k, v, float(softmax_scale), balance_alpha, grad_x)
    return o, (loss if balance_alpha is not None else None), group
