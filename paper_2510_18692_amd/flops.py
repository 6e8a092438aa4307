"""FLOP accounting for MoGA, in the convention the paper's own tables use.

Table 5's full-attention row is reproduced to three digits by
    4 * N^2 * d_model * layers + 2 * params * N
so the paper counts 4*N^2*d FLOPs per attention forward (two GEMMs, two FLOPs per
multiply-add).  Within-group attention therefore costs 4*H*D*sum_g n_g^2 forward and,
with the usual five GEMMs of the backward pass, 10*H*D*sum_g n_g^2 backward.
Sparsity in Tables 1 and 4 equals 1 - 1/M - 0.0875 for uniform groups (the constant
is the share of the static spatial-temporal group attention).
"""
from __future__ import annotations


def full_attention_model_pflops(N: int, d_model: int, layers: int, params: float) -> float:
    """Whole-model forward compute with full attention (Table 5, first row), in PFLOPs."""
    return (4.0 * N * N * d_model * layers + 2.0 * params * N) / 1e15


def moga_sparsity(M: int, static_share: float = 0.0875) -> float:
    """Sparsity of MoGA + static group attention under uniform groups (Tables 1 and 4)."""
    return 1.0 - 1.0 / M - static_share


def sum_sq(counts) -> int:
    return int(sum(int(c) * int(c) for c in counts))


def group_attn_fwd_flops(counts, H: int, D: int) -> float:
    """Within-group attention forward: 4 * H * D * sum_g n_g^2."""
    return 4.0 * H * D * sum_sq(counts)


def group_attn_bwd_flops(counts, H: int, D: int) -> float:
    """Within-group attention backward (dV, dP, dS->dQ, dK plus the recomputed S): 10 * H * D * sum n_g^2."""
    return 10.0 * H * D * sum_sq(counts)
