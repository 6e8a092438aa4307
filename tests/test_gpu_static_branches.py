"""GPU parity of the static branches of Section 3.2 (spatial-temporal groups, per-frame groups,
mean of three branches) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import moga_oracle as orc
from oracle import stga_oracle as sto
from paper_2510_18692_amd import binding as mg
from tests import parity as P

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def tdt(dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("f32", 128)])
def test_gather_with_repeats_and_its_backward(dtype, D):
    N, H, Nk = 777, 3, 2000
    g = torch.Generator().manual_seed(D)
    src = torch.randn((N, H, D), generator=g).to(tdt(dtype))
    index = torch.randint(0, N, (Nk,), generator=g, dtype=torch.int32)
    index[:5] = 7                                        # a token listed many times
    dst = mg.moga_gather_rows(src.cuda(), index.cuda())
    assert torch.equal(dst.cpu().permute(1, 0, 2), src[index.long()])
    # inverse lists by a stable sort of the index on the host
    order = np.argsort(index.numpy(), kind="stable").astype(np.int32)
    counts = np.bincount(index.numpy(), minlength=N)
    inv_cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    d_dst = torch.randn((H, Nk, D), generator=g).to(tdt(dtype))
    ref = np.zeros((N, H, D))
    np.add.at(ref, index.numpy().astype(np.int64), np.transpose(P.to64(d_dst), (1, 0, 2)))
    got = mg.moga_gather_rows_bwd(d_dst.cuda(), torch.from_numpy(inv_cu).cuda(), torch.from_numpy(order).cuda(), N)
    tol = dict(rtol=1e-6, atol=1e-6) if dtype == "f32" else dict(rtol=2 ** -8, atol=1e-6)
    np.testing.assert_allclose(P.to64(got), ref, **tol)
    assert np.all(P.to64(got)[counts == 0] == 0)
    base = torch.randn((N, H, D), generator=g).to(tdt(dtype))
    acc = base.clone().cuda()
    mg.moga_gather_rows_bwd(d_dst.cuda(), torch.from_numpy(inv_cu).cuda(), torch.from_numpy(order).cuda(), N, d_src=acc)
    np.testing.assert_allclose(P.to64(acc), P.to64(base) + ref, rtol=tol["rtol"], atol=2e-2 if dtype == "bf16" else 1e-5)


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("f32", 128)])
def test_one_pass_sum_of_the_three_branch_gradients(dtype, D):
    """moga_gather3_bwd against the sum written out on the host, and against the three calls it replaces."""
    N, H, Nk = 1003, 3, 1400
    g = torch.Generator().manual_seed(5 + D)
    g_m, g_f = (torch.randn((H, N, D), generator=g).to(tdt(dtype)) for _ in range(2))
    g_s = torch.randn((H, Nk, D), generator=g).to(tdt(dtype))
    perm = torch.randperm(N, generator=g).to(torch.int32)
    inv_m = torch.empty_like(perm)
    inv_m[perm.long()] = torch.arange(N, dtype=torch.int32)
    index = torch.randint(0, N, (Nk,), generator=g, dtype=torch.int32)      # token listed by slot j
    index[:4] = 9                                                          # a token with several slots
    index[index == 11] = 12                                                # a token with none
    order = np.argsort(index.numpy(), kind="stable").astype(np.int32)
    counts = np.bincount(index.numpy(), minlength=N)
    inv_cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    tok = lambda a: np.transpose(P.to64(a), (1, 0, 2))
    ref = tok(g_m)[inv_m.numpy()] + tok(g_f)
    np.add.at(ref, index.numpy().astype(np.int64), tok(g_s))
    cu, sl = torch.from_numpy(inv_cu).cuda(), torch.from_numpy(order).cuda()
    got = mg.moga_gather3_bwd(g_m.cuda(), inv_m.cuda(), g_s.cuda(), cu, sl, g_f.cuda())
    torch.cuda.synchronize()
    tol = dict(rtol=1e-6, atol=1e-6) if dtype == "f32" else dict(rtol=2 ** -8, atol=1e-6)   # one rounding
    np.testing.assert_allclose(P.to64(got), ref, **tol)
    # the calls it replaces round after every step (bf16): same result within those roundings
    d, _, _ = mg.moga_permute_bwd(g_m.cuda(), g_m.cuda(), g_m.cuda(), perm.cuda())
    mg.moga_gather_rows_bwd(g_s.cuda(), cu, sl, N, d_src=d)
    ident = torch.arange(N + 1, dtype=torch.int32).cuda()
    mg.moga_gather_rows_bwd(g_f.cuda(), ident, ident[:N], N, d_src=d)
    np.testing.assert_allclose(P.to64(d), P.to64(got), rtol=2 ** -6 if dtype == "bf16" else 1e-5,
                               atol=3e-2 if dtype == "bf16" else 1e-5)


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_merge_of_three_branches_and_its_backward(dtype, D):
    N, H = 1000, 5
    g = torch.Generator().manual_seed(11 + D)
    a_m, a_s, a_f = (torch.randn((H, N, D), generator=g).to(tdt(dtype)) for _ in range(3))
    inv_m = torch.randperm(N, generator=g).to(torch.int32)
    inv_s = torch.randperm(N, generator=g).to(torch.int32)
    gate = torch.rand(N, generator=g)
    d_o = torch.randn((N, H, D), generator=g).to(tdt(dtype))
    tok = lambda a, inv: np.transpose(P.to64(a), (1, 0, 2))[inv.numpy()] if inv is not None else np.transpose(P.to64(a), (1, 0, 2))
    ref = (P.to64(gate)[:, None, None] * tok(a_m, inv_m) + tok(a_s, inv_s) + tok(a_f, None)) / 3
    o = mg.moga_merge3_fwd(a_m.cuda(), a_s.cuda(), a_f.cuda(), inv_m.cuda(), inv_s.cuda(), None, gate.cuda())
    np.testing.assert_allclose(P.to64(o), ref, rtol=2 ** -8 if dtype == "bf16" else 1e-6, atol=1e-6)
    d_m, d_s, d_f, d_gate = mg.moga_merge3_bwd(d_o.cuda(), a_m.cuda(), inv_m.cuda(), inv_s.cuda(), None, gate.cuda())
    dO = P.to64(d_o)
    rt = 2 ** -8 if dtype == "bf16" else 1e-6
    ref_m = np.empty((N, H, D)); ref_m[inv_m.numpy()] = dO * P.to64(gate)[:, None, None] / 3
    ref_s = np.empty((N, H, D)); ref_s[inv_s.numpy()] = dO / 3
    np.testing.assert_allclose(P.unhat(d_m), ref_m, rtol=rt, atol=1e-7)
    np.testing.assert_allclose(P.unhat(d_s), ref_s, rtol=rt, atol=1e-7)
    np.testing.assert_allclose(P.unhat(d_f), dO / 3, rtol=rt, atol=1e-7)
    ref_g = (dO * tok(a_m, inv_m)).sum(axis=(1, 2)) / 3
    np.testing.assert_allclose(P.to64(d_gate), ref_g, rtol=1e-4, atol=1e-3)


def visual_block_gpu(inp, grid, wh, ww, tg, shot, scale):
    """The three-branch block through the C ABI, forward and backward."""
    T, Hh, Ww = grid
    si = mg.moga_stga_build_index(T, Hh, Ww, wh, ww, tg, shot)
    fwd = mg.visual_forward(inp["X"], inp["W"], inp["Q"], inp["K"], inp["V"], scale, grid, si)
    bwd = mg.visual_backward(fwd, inp["X"], inp["W"], inp["dO"], scale)
    torch.cuda.synchronize()
    return fwd, bwd


@pytest.mark.parametrize("dtype,D,H,d_model", [("f32", 64, 2, 128), ("bf16", 128, 3, 256)])
def test_three_branch_block_forward_and_backward(dtype, D, H, d_model):
    T, Hh, Ww, wh, ww, tg, M = 9, 8, 12, 4, 6, 2, 4
    shot = [0, 0, 0, 0, 1, 1, 1, 2, 2]
    N = T * Hh * Ww
    say(f"three-branch block {dtype}: N={N}")
    g = torch.Generator().manual_seed(77)
    X = torch.randn((N, d_model), generator=g).to(tdt(dtype))
    W = torch.randn((M, d_model), generator=g) * (2.0 / d_model ** 0.5)
    Q, K, V, dO = (torch.randn((N, H, D), generator=g).to(tdt(dtype)) for _ in range(4))
    scale = D ** -0.5
    X64, W64, Q64, K64, V64, dO64 = (P.to64(t) for t in (X, W, Q, K, V, dO))
    ref = sto.visual_attention(X64, W64, Q64, K64, V64, scale, (T, Hh, Ww), wh, ww, tg, shot)
    refb = sto.visual_attention_bwd(ref, X64, W64, Q64, K64, V64, dO64, scale)
    inp = {k: t.cuda() for k, t in (("X", X), ("W", W), ("Q", Q), ("K", K), ("V", V), ("dO", dO))}
    fwd, bwd = visual_block_gpu(inp, (T, Hh, Ww), wh, ww, tg, shot, scale)
    assert not P.check_assignment(fwd["group"].cpu().numpy(), ref["moga"])
    if dtype == "f32":
        say("  O", P.assert_close_f32(P.to64(fwd["o"]), ref["O"], "O"))
        for n, k in (("dQ", "d_q"), ("dK", "d_k"), ("dV", "d_v"), ("dW", "d_w")):
            say(f"  {n}", P.assert_close_f32(P.to64(bwd[k]), refb[n], n))
    else:
        say("  O", P.assert_close_bf16(P.to64(fwd["o"]), ref["O"], "O"))
        for n, k in (("dQ", "d_q"), ("dK", "d_k"), ("dV", "d_v")):
            rm, rl = P.rel_max(P.to64(bwd[k]), refb[n]), P.rel_l2(P.to64(bwd[k]), refb[n])
            say(f"  {n} rel max {rm:.2e} l2 {rl:.2e}")
            assert rm <= P.BF16_REL_MAX and rl <= P.BF16_REL_L2
        rl = P.rel_l2(P.to64(bwd["d_w"]), refb["dW"])
        say(f"  dW l2 {rl:.2e}")
        assert rl <= 5e-3
