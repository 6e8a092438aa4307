"""Seeded random group-size mixes through the attention calls (forward, backward, separate
query/key lists) against the oracle: many tile-boundary combinations in one run."""
import numpy as np
import pytest
import torch

from oracle import stga_oracle as sto
from paper_2510_18692_amd import binding as mg
from tests import parity as P

pytestmark = pytest.mark.gpu


def draw_sizes(rng, G, hi):
    """Group sizes with many tile-edge values, empties and a heavy tail."""
    edges = np.array([0, 1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513])
    pick = rng.random(G)
    out = np.where(pick < 0.5, rng.choice(edges, G), rng.integers(0, hi, G))
    return out.astype(int).tolist()


@pytest.mark.parametrize("seed", list(range(12)))
def test_random_group_mixes_forward_and_backward(seed):
    rng = np.random.default_rng(1000 + seed)
    G = int(rng.integers(1, 40))
    H = int(rng.integers(1, 4))
    nq = draw_sizes(rng, G, 700)
    same = seed % 3 != 0
    nk = list(nq) if same else [int(max(0, n + rng.integers(-20, 200))) for n in nq]
    if sum(nq) == 0:
        nq[0] = 5
        nk[0] = 5 if same else nk[0]
    print(f"seed {seed}: G={G} H={H} same_lists={same} Nq={sum(nq)} Nk={sum(nk)}", flush=True)
    D, scale = 128, 128 ** -0.5
    g = torch.Generator().manual_seed(seed)
    Nq, Nk = sum(nq), sum(nk)
    q, dA = (torch.randn((Nq, H, D), generator=g).bfloat16() for _ in range(2))
    k, v = (torch.randn((Nk, H, D), generator=g).bfloat16() for _ in range(2))
    cu_q = np.concatenate([[0], np.cumsum(nq)]).astype(np.int32)
    cu_k = np.concatenate([[0], np.cumsum(nk)]).astype(np.int32)
    q64, k64, v64, dA64 = (P.to64(t) for t in (q, k, v, dA))
    A, lse = sto.varlen_attention(q64, k64, v64, np.arange(Nq), cu_q, np.arange(Nk), cu_k, scale)
    dQ, dK, dV = sto.varlen_attention_bwd(q64, k64, v64, dA64, np.arange(Nq), cu_q, np.arange(Nk), cu_k, scale)
    tohat = lambda t: t.permute(1, 0, 2).contiguous().cuda()
    cq, ck = torch.from_numpy(cu_q).cuda(), torch.from_numpy(cu_k).cuda()
    if same and G <= 256:
        oh, lse_g = mg.moga_group_attn_fwd(tohat(q), tohat(k), tohat(v), cq, scale)
    else:
        oh, lse_g = mg.moga_varlen_attn_fwd(tohat(q), tohat(k), tohat(v), cq, ck, scale)
    P.assert_close_bf16(P.unhat(oh), A, "O")
    fin = np.isfinite(lse)
    np.testing.assert_allclose(P.to64(lse_g).T[fin], lse[fin], rtol=1e-3, atol=2e-3)
    oh_ref = torch.from_numpy(P.hat(A)).bfloat16().cuda()
    lse_ref = torch.from_numpy(np.ascontiguousarray(lse.T)).float().cuda()
    if same and G <= 256:
        grads = mg.moga_group_attn_bwd(tohat(dA), tohat(q), tohat(k), tohat(v), oh_ref, lse_ref, cq, scale)
    else:
        grads = mg.moga_varlen_attn_bwd(tohat(dA), tohat(q), tohat(k), tohat(v), oh_ref, lse_ref, cq, ck, scale)
    torch.cuda.synchronize()
    for name, got, ref in zip(("dQ", "dK", "dV"), grads, (dQ, dK, dV)):
        gg = P.unhat(got)
        assert np.all(np.isfinite(gg)), name
        if ref.size and np.abs(ref).max() > 0:
            rm, rl = P.rel_max(gg, ref), P.rel_l2(gg, ref)
            assert rm <= P.BF16_REL_MAX and rl <= P.BF16_REL_L2, (name, rm, rl)
