"""GPU parity of the forward path against the CPU oracle, call by call through the C ABI.

Every stage is fed inputs made by the seeded generators or by the oracle's upstream stage
(never by another GPU stage), and compared element by element.
"""
import math

import numpy as np
import pytest
import torch

from oracle import moga_oracle as orc
from paper_2510_18692_amd import binding as mg
from paper_2510_18692_amd import workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------------------------------
# router
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,d,M,dtype,bias", [
    (4096, 128, 8, "f32", False),      # C1 shape, generic kernel
    (1000, 96, 5, "f32", True),        # ragged, bias
    (333, 128, 40, "f32", False),      # more than 32 groups
    (257, 200, 256, "bf16", False),    # generic bf16 (d not a multiple of 64), max groups
    (4096, 1536, 8, "bf16", False),    # MFMA path, C2 widths
    (1001, 512, 5, "bf16", True),      # MFMA path, ragged tokens, M not a multiple of 4, bias
    (130, 64, 32, "bf16", False),      # MFMA path, one k block, full 32 rows
    (70000, 320, 20, "bf16", False),   # MFMA path with two token tiles per wave, ragged tail
    (1, 64, 1, "bf16", False),         # single token, single group
    (300, 192, 12, "bf16", True),      # MFMA path, three k blocks: the second weight chunk is half full
    (515, 128, 32, "bf16", False),     # MFMA path, exactly one weight chunk
])
def test_route_matches_oracle(N, d, M, dtype, bias):
    say(f"route N={N} d={d} M={M} {dtype} bias={bias}")
    g = torch.Generator().manual_seed(N + d + M)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = torch.randn((N, d), generator=g).to(tdt)
    w = torch.randn((M, d), generator=g) * (2.0 / math.sqrt(d))
    b = torch.randn(M, generator=g) if bias else None
    rt = orc.route(P.to64(x), P.to64(w), None if b is None else P.to64(b))
    group, gate, probs, logits = mg.moga_route(x.cuda(), w.cuda(), None if b is None else b.cuda(),
                                               want_probs=True, want_logits=True)
    torch.cuda.synchronize()
    err = np.abs(P.to64(logits) - rt["r64"]).max()
    say(f"  max |logit_gpu - logit_oracle| = {err:.3e}")
    assert err < 2e-5
    bad = P.check_assignment(group.cpu().numpy(), rt)
    keep = np.ones(N, bool)
    keep[[m[0] for m in bad]] = False
    np.testing.assert_allclose(P.to64(gate)[keep], rt["gate"][keep], rtol=2e-5)
    np.testing.assert_allclose(P.to64(probs)[keep], rt["probs"][keep], rtol=1e-4, atol=1e-7)
    np.testing.assert_allclose(P.to64(probs).sum(1), 1.0, rtol=1e-5)


def test_route_zero_weight_sends_every_token_to_group_zero():
    x = torch.randn(300, 128).bfloat16().cuda()
    w = torch.zeros(8, 128).cuda()
    group, gate, probs, _ = mg.moga_route(x, w)
    assert torch.all(group == 0)
    np.testing.assert_allclose(P.to64(gate), 1 / 8, rtol=1e-6)
    xf = torch.randn(300, 100).cuda()
    group, gate, _, _ = mg.moga_route(xf, torch.zeros(7, 100).cuda())
    assert torch.all(group == 0)
    np.testing.assert_allclose(P.to64(gate), 1 / 7, rtol=1e-6)


# ------------------------------------------------------------------------------------------
# permutation + gather
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,M", [(0, 4), (1, 1), (63, 3), (64, 8), (513, 5), (4096, 8), (10007, 256),
                                 (99840, 16), (580320, 32), (5000000, 20)])
def test_permutation_integers_are_bit_exact(N, M):
    say(f"permute ints N={N} M={M}")
    rng = np.random.default_rng(N + M)
    if N > 100:
        w = (np.arange(1, M + 1) ** -1.1)
        group = rng.choice(M, size=N, p=w / w.sum()).astype(np.int32)
        if M > 2:
            group[group == 1] = 0          # an empty group
    else:
        group = rng.integers(0, M, size=N).astype(np.int32)
    ref = orc.permute_index(group, M)
    out = mg.moga_permute(torch.from_numpy(group).cuda(), M)
    torch.cuda.synchronize()
    for name in ("counts", "cu_seqlens", "perm", "inv_perm"):
        assert np.array_equal(out[name].cpu().numpy(), ref[name]), name
    assert int(out["max_seqlen"].item()) == int(ref["max_seqlen"])


def test_permutation_is_deterministic_and_ignores_workspace_contents():
    group = torch.randint(0, 12, (70001,), dtype=torch.int32).cuda()
    a = mg.moga_permute(group, 12)
    torch.empty(1 << 20, dtype=torch.int32, device="cuda").fill_(-559038737)   # poison freed memory
    b = mg.moga_permute(group, 12)
    assert torch.equal(a["perm"], b["perm"]) and torch.equal(a["cu_seqlens"], b["cu_seqlens"])


def test_out_of_range_group_ids_are_clamped():
    group = torch.tensor([5, -3, 1, 99, 0], dtype=torch.int32).cuda()
    out = mg.moga_permute(group, 4)
    assert out["counts"].tolist() == [2, 1, 0, 2]
    assert out["perm"].tolist() == [1, 4, 2, 0, 3]


@pytest.mark.parametrize("N,H,D,M,dtype", [(4096, 2, 64, 8, "f32"), (1000, 3, 128, 5, "f32"),
                                           (3001, 12, 128, 8, "bf16"), (17, 40, 128, 16, "bf16")])
def test_gather_puts_rows_in_group_contiguous_head_major_order(N, H, D, M, dtype):
    say(f"gather N={N} H={H} D={D} {dtype}")
    g = torch.Generator().manual_seed(N)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    q, k, v = (torch.randn((N, H, D), generator=g).to(tdt) for _ in range(3))
    group = torch.randint(0, M, (N,), generator=g, dtype=torch.int32)
    ref = orc.permute_index(group.numpy(), M)
    out = mg.moga_permute(group.cuda(), M, q.cuda(), k.cuda(), v.cuda())
    torch.cuda.synchronize()
    perm = torch.from_numpy(ref["perm"].astype(np.int64))
    for name, t in (("qh", q), ("kh", k), ("vh", v)):
        expect = t[perm].permute(1, 0, 2).contiguous()
        assert torch.equal(out[name].cpu(), expect), name      # a copy: bit-exact


# ------------------------------------------------------------------------------------------
# attention inside groups
# ------------------------------------------------------------------------------------------
def attn_case(sizes, H, D, dtype, seed, scale=None, peaked=False):
    """Hand-assigned group sizes (sorted order): returns oracle inputs and device tensors."""
    N = int(sum(sizes))
    g = torch.Generator().manual_seed(seed)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    q, k, v = (torch.randn((N, H, D), generator=g).to(tdt) for _ in range(3))
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    if peaked:
        # Clusters of 8 consecutive rows of a group share a direction b: q = (b + e_q) / sqrt(2),
        # k = (b + e_k) / sqrt(2), still unit variance.  A query's score is about 5.7 +- 1 on the 8
        # keys of its cluster and N(0, 1) elsewhere, so a handful of keys share most of the softmax
        # mass with unequal weights: |O| is of the order of |V| and the rounding of P matters.
        qq, kk = q.float(), k.float()
        for s, e in zip(cu[:-1], cu[1:]):
            n = int(e - s)
            base = torch.randn(((n + 7) // 8, H, D), generator=g).repeat_interleave(8, dim=0)[:n]
            qq[s:e] = (base + qq[s:e]) / math.sqrt(2.0)
            kk[s:e] = (base + kk[s:e]) / math.sqrt(2.0)
        q, k = qq.to(tdt), kk.to(tdt)
    scale = scale if scale is not None else D ** -0.5
    return q, k, v, cu, scale


@pytest.mark.parametrize("sizes,H,D,dtype", [
    ([512] * 8, 2, 64, "f32"),                          # C1 shape in sorted order
    ([1, 0, 65, 130, 31, 0, 64, 200], 2, 64, "f32"),    # ragged, empty groups, a group of one
    ([100, 3], 1, 128, "f32"),
    ([300, 0, 1, 129, 257, 64, 2, 511], 3, 128, "bf16"),  # crosses 64/128/256 tile edges
    ([4095, 4096, 17], 2, 128, "bf16"),
    ([40], 1, 128, "bf16"),
    ([288, 289, 319, 320, 321, 352, 575, 576, 577, 33, 32, 31, 63, 64, 65, 95, 96, 97, 127, 128, 1, 2], 1, 128, "bf16"),
])
def test_group_attention_forward_matches_oracle(sizes, H, D, dtype):
    say(f"attn fwd sizes={sizes} H={H} D={D} {dtype}")
    q, k, v, cu, scale = attn_case(sizes, H, D, dtype, seed=len(sizes) + D)
    A, lse = orc.group_attention(P.to64(q), P.to64(k), P.to64(v), cu, scale)
    tohat = lambda t: t.permute(1, 0, 2).contiguous().cuda()
    oh, lse_g = mg.moga_group_attn_fwd(tohat(q), tohat(k), tohat(v), torch.from_numpy(cu).cuda(), scale)
    torch.cuda.synchronize()
    got = P.unhat(oh)
    if dtype == "f32":
        e = P.assert_close_f32(got, A, "attention output")
        np.testing.assert_allclose(P.to64(lse_g).T, lse, rtol=1e-5, atol=1e-5)
    else:
        e = P.assert_close_bf16(got, A, "attention output")
        np.testing.assert_allclose(P.to64(lse_g).T, lse, rtol=1e-3, atol=2e-3)
    say(f"  error {e}")
    assert np.all(np.isfinite(got))


def test_group_attention_bf16_peaked_rows_have_teeth():
    """A handful of keys share each query's softmax mass, so |O| ~ |V| and P's rounding to bf16
    shows: the stated 2e-2 max-abs bound is not vacuous here (and the softmax is not one-hot)."""
    sizes = [700, 300, 1000, 8, 3]
    q, k, v, cu, scale = attn_case(sizes, 2, 128, "bf16", seed=5, peaked=True)
    A, _ = orc.group_attention(P.to64(q), P.to64(k), P.to64(v), cu, scale)
    # shape of the softmax in the largest group, head 0 (a property of the input, not a reference)
    s0, e0 = int(cu[2]), int(cu[3])
    S = scale * P.to64(q)[s0:e0, 0] @ P.to64(k)[s0:e0, 0].T
    Pm = np.exp(S - S.max(1, keepdims=True))
    Pm /= Pm.sum(1, keepdims=True)
    top, top8 = np.median(Pm.max(1)), np.median(np.sort(Pm, 1)[:, -8:].sum(1))
    say(f"  peaked case: median top-1 prob {top:.3f}, median top-8 mass {top8:.3f}, max|A| {np.abs(A).max():.2f}, "
        f"rms A {np.sqrt((A ** 2).mean()):.3f}")
    assert 0.05 < top < 0.8 and top8 > 0.5          # peaked, but several keys share the mass
    assert np.sqrt((A ** 2).mean()) > 0.25          # outputs of the order of the values
    tohat = lambda t: t.permute(1, 0, 2).contiguous().cuda()
    oh, _ = mg.moga_group_attn_fwd(tohat(q), tohat(k), tohat(v), torch.from_numpy(cu).cuda(), scale)
    say("  peaked error", P.assert_close_bf16(P.unhat(oh), A, "peaked attention output"))   # the stated 2e-2


def test_group_attention_constant_values_return_the_value():
    """V_j = v for all j: every softmax average is v itself, for any group sizes."""
    sizes = [70, 0, 200, 1]
    q, k, v, cu, scale = attn_case(sizes, 2, 128, "bf16", seed=9)
    v[:] = torch.randn(2, 128).bfloat16()
    tohat = lambda t: t.permute(1, 0, 2).contiguous().cuda()
    oh, _ = mg.moga_group_attn_fwd(tohat(q), tohat(k), tohat(v), torch.from_numpy(cu).cuda(), scale)
    np.testing.assert_allclose(P.unhat(oh), P.to64(v), atol=2e-2, rtol=1e-2)


# ------------------------------------------------------------------------------------------
# scatter + gate
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,H,D,dtype,gated", [(4096, 2, 64, "f32", True), (999, 3, 128, "f32", False),
                                               (3001, 12, 128, "bf16", True)])
def test_unpermute_scatters_and_scales_by_gate(N, H, D, dtype, gated):
    g = torch.Generator().manual_seed(N + 1)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    oh = torch.randn((H, N, D), generator=g).to(tdt)
    perm = torch.randperm(N, generator=g).to(torch.int32)
    gate = torch.rand(N, generator=g) if gated else None
    ref = orc.unpermute(np.transpose(P.to64(oh), (1, 0, 2)), perm.numpy(), None if gate is None else P.to64(gate))
    o = mg.moga_unpermute(oh.cuda(), perm.cuda(), None if gate is None else gate.cuda())
    torch.cuda.synchronize()
    if dtype == "f32":
        np.testing.assert_allclose(P.to64(o), ref, rtol=2e-7, atol=0)
    else:
        np.testing.assert_allclose(P.to64(o), ref, rtol=2 ** -8, atol=0)   # one bf16 rounding


# ------------------------------------------------------------------------------------------
# whole forward
# ------------------------------------------------------------------------------------------
def run_forward(w, device_inputs=None):
    inp = wl.make_inputs(w, "cpu")
    f = orc.moga_forward(P.to64(inp["X"]), P.to64(inp["W"]), P.to64(inp["Q"]), P.to64(inp["K"]),
                         P.to64(inp["V"]), w.scale)
    d = {k: inp[k].cuda() for k in ("X", "W", "Q", "K", "V")}
    out = mg.moga_forward(d["X"], d["W"], d["Q"], d["K"], d["V"], w.scale)
    torch.cuda.synchronize()
    return inp, f, out


def test_config1_fp32_forward_every_element():
    w = wl.WORKLOADS["C1"]
    say("C1 full forward")
    inp, f, out = run_forward(w)
    bad = P.check_assignment(out["group"].cpu().numpy(), f)
    assert not bad, "fp32 config: assignments must agree"
    for name in ("counts", "cu_seqlens", "perm", "inv_perm"):
        assert np.array_equal(out[name].cpu().numpy(), f[name]), name
    say("  counts", f["counts"].tolist())
    P.assert_close_f32(P.unhat(out["oh"]), f["A"], "A")
    e = P.assert_close_f32(P.to64(out["o"]), f["O"], "O")
    np.testing.assert_allclose(P.to64(out["gate"]), f["gate"], rtol=1e-5)
    say(f"  O rel err {e:.3e}")


@pytest.mark.timeout(600)
def test_config2_bf16_forward_every_element():
    """Configuration 2 at its stated size: N = 32,760 (21 frames), 12 heads, head_dim 128,
    d_model 1536, M = 8; every output element against the full oracle."""
    w = wl.WORKLOADS["C2"]
    say(f"C2 full forward: N={w.N} H={w.H}")
    inp, f, out = run_forward(w)
    bad = P.check_assignment(out["group"].cpu().numpy(), f)
    say(f"  argmax mismatches (margin < 1e-5 only): {len(bad)}; counts {f['counts'].tolist()}")
    if not bad:
        for name in ("counts", "cu_seqlens", "perm", "inv_perm"):
            assert np.array_equal(out[name].cpu().numpy(), f[name]), name
        e = P.assert_close_bf16(P.unhat(out["oh"]), f["A"], "A")
        say(f"  A (ungated, sorted order) error {e}")
    keep = np.ones(w.N, bool)
    keep[[m[0] for m in bad]] = False
    np.testing.assert_allclose(P.to64(out["gate"])[keep], f["gate"][keep], rtol=3e-5)
    say("  O error", P.assert_close_bf16(P.to64(out["o"])[keep], f["O"][keep], "O"))


def test_single_group_is_full_attention_on_the_gpu():
    w = wl.scaled(wl.WORKLOADS["C1"], N=700, M=1)
    inp, f, out = run_forward(w)
    assert torch.all(out["group"] == 0) and torch.all(out["gate"] == 1.0)
    full, _ = orc.softmax_attention(P.to64(inp["Q"])[:, 0], P.to64(inp["K"])[:, 0], P.to64(inp["V"])[:, 0], w.scale)
    P.assert_close_f32(P.to64(out["o"])[:, 0], full, "M=1 vs full attention")
