"""FLOP-accounting convention pinned to the numbers the paper prints (no GPU)."""
import os

import pytest

from paper_2510_18692_amd import flops

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [tuple(float(x) for x in line.split()) for line in f if line.strip() and not line.startswith("#")]


def test_full_attention_row_of_table5_fixes_four_n_squared_d_per_attention():
    for n, printed in rows("table5_full_attention_pflops.txt"):
        got = flops.full_attention_model_pflops(int(n), 1536, 30, 1.3e9)
        assert abs(got - printed) < 0.01, (n, got, printed)   # printed to 2 decimals
        # a 2*N^2*d convention (one FLOP per multiply-add) would be off by almost 2x
        half = (2.0 * n * n * 1536 * 30 + 2 * 1.3e9 * n) / 1e15
        assert abs(half - printed) > 0.05 * printed


def test_sparsity_closed_form_matches_printed_values():
    for m, printed in rows("sparsity_vs_groups.txt"):
        assert abs(100 * flops.moga_sparsity(int(m)) - printed) < 1e-9


def test_effective_flops_formulas():
    counts = [3, 0, 5]
    assert flops.sum_sq(counts) == 34
    assert flops.group_attn_fwd_flops(counts, 2, 8) == 4 * 2 * 8 * 34
    assert flops.group_attn_bwd_flops(counts, 2, 8) == 10 * 2 * 8 * 34
    # uniform groups: cost is 1/M of full attention (Section 3.2 complexity claim)
    n, m = 1200, 4
    assert flops.group_attn_fwd_flops([n // m] * m, 1, 1) == pytest.approx(4.0 * n * n / m)
