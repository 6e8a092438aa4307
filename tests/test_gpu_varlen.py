"""GPU parity of attention inside static groups with separately listed queries and keys
(moga_varlen_attn_fwd / _bwd) against the CPU oracle, element by element through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import stga_oracle as sto
from paper_2510_18692_amd import binding as mg
from tests import parity as P

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def tdt(dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def make_case(nq_list, nk_list, H, D, dtype, seed):
    Nq, Nk = int(sum(nq_list)), int(sum(nk_list))
    g = torch.Generator().manual_seed(seed)
    q, dA = (torch.randn((Nq, H, D), generator=g).to(tdt(dtype)) for _ in range(2))
    k, v = (torch.randn((Nk, H, D), generator=g).to(tdt(dtype)) for _ in range(2))
    cu_q = np.concatenate([[0], np.cumsum(nq_list)]).astype(np.int32)
    cu_k = np.concatenate([[0], np.cumsum(nk_list)]).astype(np.int32)
    return q, k, v, dA, cu_q, cu_k


def run_case(nq_list, nk_list, H, D, dtype, seed, backward=True):
    q, k, v, dA, cu_q, cu_k = make_case(nq_list, nk_list, H, D, dtype, seed)
    Nq, Nk = q.shape[0], k.shape[0]
    scale = D ** -0.5
    qi, ki = np.arange(Nq), np.arange(Nk)
    q64, k64, v64, dA64 = (P.to64(t) for t in (q, k, v, dA))
    A, lse = sto.varlen_attention(q64, k64, v64, qi, cu_q, ki, cu_k, scale)
    tohat = lambda t: t.permute(1, 0, 2).contiguous().cuda()
    cuq_t, cuk_t = torch.from_numpy(cu_q).cuda(), torch.from_numpy(cu_k).cuda()
    oh, lse_g = mg.moga_varlen_attn_fwd(tohat(q), tohat(k), tohat(v), cuq_t, cuk_t, scale)
    torch.cuda.synchronize()
    got = P.unhat(oh)
    if dtype == "f32":
        e = P.assert_close_f32(got, A, "varlen attention")
    else:
        e = P.assert_close_bf16(got, A, "varlen attention")
    lse_got = P.to64(lse_g).T
    fin = np.isfinite(lse)
    np.testing.assert_allclose(lse_got[fin], lse[fin], rtol=1e-3 if dtype == "bf16" else 1e-5, atol=2e-3 if dtype == "bf16" else 1e-5)
    assert np.all(lse_got[~fin] == -np.inf) and np.all(got[~fin] == 0)
    say(f"  forward error {e}")
    if not backward:
        return
    dQ, dK, dV = sto.varlen_attention_bwd(q64, k64, v64, dA64, qi, cu_q, ki, cu_k, scale)
    oh_ref = torch.from_numpy(P.hat(A)).to(tdt(dtype)).cuda()
    lse_ref = torch.from_numpy(np.ascontiguousarray(lse.T)).float().cuda()
    d_qh, d_kh, d_vh = mg.moga_varlen_attn_bwd(tohat(dA), tohat(q), tohat(k), tohat(v), oh_ref, lse_ref, cuq_t, cuk_t, scale)
    torch.cuda.synchronize()
    for name, got_t, ref in (("dQ", d_qh, dQ), ("dK", d_kh, dK), ("dV", d_vh, dV)):
        gg = P.unhat(got_t)
        assert np.all(np.isfinite(gg)), name
        if ref.size == 0:
            continue
        if dtype == "f32":
            e = P.assert_close_f32(gg, ref, name)
        else:
            rm, rl = P.rel_max(gg, ref), P.rel_l2(gg, ref)
            assert rm <= P.BF16_REL_MAX and rl <= P.BF16_REL_L2, (name, rm, rl)
            e = (rm, rl)
        say(f"  {name} error {e}")
        # rows of a group whose other side is empty are exactly zero
        mine, other = (cu_q, cu_k) if name == "dQ" else (cu_k, cu_q)
        for g in range(len(cu_q) - 1):
            if other[g + 1] == other[g]:
                assert np.all(gg[mine[g]:mine[g + 1]] == 0), (name, g)


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_more_keys_than_queries_and_empty_sides(dtype, D):
    say(f"varlen {dtype}")
    run_case([300, 0, 64, 1, 257, 129, 31], [420, 50, 0, 1, 33, 700, 95], 2, D, dtype, seed=3)


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_many_small_groups_use_the_presummed_tile_index(dtype, D):
    rng = np.random.default_rng(5)
    G = 700                                  # more groups than the router path supports
    nq = rng.integers(0, 48, G)
    nk = nq + rng.integers(0, 24, G)
    nk[rng.integers(0, G, 20)] = 0           # a few groups whose queries have no keys
    say(f"varlen many groups {dtype}: Nq={nq.sum()} Nk={nk.sum()}")
    run_case(nq.tolist(), nk.tolist(), 2, D, dtype, seed=6)


def test_equal_lists_reproduce_group_attention_bit_for_bit():
    sizes = [513, 0, 77, 1024, 3]
    q, k, v, dA, cu, _ = make_case(sizes, sizes, 3, 128, "bf16", seed=8)
    tohat = lambda t: t.permute(1, 0, 2).contiguous().cuda()
    cu_t = torch.from_numpy(cu).cuda()
    oh1, lse1 = mg.moga_group_attn_fwd(tohat(q), tohat(k), tohat(v), cu_t, 0.09)
    oh2, lse2 = mg.moga_varlen_attn_fwd(tohat(q), tohat(k), tohat(v), cu_t, cu_t, 0.09)
    assert torch.equal(oh1, oh2) and torch.equal(lse1, lse2)
    g1 = mg.moga_group_attn_bwd(tohat(dA), tohat(q), tohat(k), tohat(v), oh1, lse1, cu_t, 0.09)
    g2 = mg.moga_varlen_attn_bwd(tohat(dA), tohat(q), tohat(k), tohat(v), oh1, lse1, cu_t, cu_t, 0.09)
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)


def test_long_keys_short_queries_bf16():
    run_case([40, 700], [2100, 1300], 1, 128, "bf16", seed=9)


def test_all_queries_without_keys():
    q, k, v, dA, cu_q, cu_k = make_case([100, 30], [0, 0], 2, 128, "bf16", seed=10)
    tohat = lambda t: t.permute(1, 0, 2).contiguous().cuda()
    oh, lse = mg.moga_varlen_attn_fwd(tohat(q), tohat(k), tohat(v), torch.from_numpy(cu_q).cuda(),
                                      torch.from_numpy(cu_k).cuda(), 0.1)
    assert torch.all(oh == 0) and torch.all(lse == -float("inf"))
