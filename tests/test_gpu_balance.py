"""GPU parity of the group balancing loss (Eqs. 6-8) and its gate gradient against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import moga_oracle as orc
from paper_2510_18692_amd import binding as mg
from paper_2510_18692_amd import workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu

ALPHA = 0.1   # the paper's training setup


def say(*a):
    print(*a, flush=True)


def case(N, M, seed, skew=False):
    g = torch.Generator().manual_seed(seed)
    if skew:      # most tokens in a few groups, several groups empty
        w = torch.zeros(M)
        w[: max(1, M // 3)] = torch.rand(max(1, M // 3), generator=g) + 0.05
        group = torch.multinomial(w, N, replacement=True, generator=g).to(torch.int32)
    else:
        group = torch.randint(0, M, (N,), generator=g, dtype=torch.int32)
    gate = (torch.rand(N, generator=g) * (1 - 1.0 / M) + 1.0 / M).float()
    return group, gate


@pytest.mark.parametrize("N,M,skew", [(4096, 8, False), (100001, 32, False), (100001, 32, True), (5, 256, False),
                                      (1, 1, False), (70000, 16, True), (1000, 200, False)])
def test_balance_loss_matches_oracle(N, M, skew):
    say(f"balance loss N={N} M={M} skew={skew}")
    group, gate = case(N, M, seed=N + M, skew=skew)
    L, F, Pm = orc.balance_loss(group.numpy(), P.to64(gate), M, ALPHA)
    loss, frac, prob = mg.moga_balance_loss(group.cuda(), gate.cuda(), M, ALPHA)
    loss2, frac2, prob2 = mg.moga_balance_loss(group.cuda(), gate.cuda(), M, ALPHA)
    torch.cuda.synchronize()
    np.testing.assert_allclose(P.to64(frac), F, rtol=1e-6, atol=0)
    np.testing.assert_allclose(P.to64(prob), Pm, rtol=1e-6, atol=0)
    np.testing.assert_allclose(float(loss.item()), L, rtol=1e-6)
    say(f"  loss {float(loss.item()):.8f} vs {L:.8f}")
    # integer accumulation: the result does not depend on the order of the atomics
    assert torch.equal(loss, loss2) and torch.equal(frac, frac2) and torch.equal(prob, prob2)


def test_uniform_assignment_with_confident_router_gives_alpha():
    """Perfect balance and gate = 1 for every token: F_i = P_i = 1/M, so L = alpha (metric L/alpha = 1)."""
    N, M = 32 * 1000, 32
    group = (torch.arange(N) % M).to(torch.int32).cuda()
    loss, frac, prob = mg.moga_balance_loss(group, torch.ones(N).cuda(), M, ALPHA)
    assert abs(float(loss.item()) - ALPHA) <= 1e-7
    assert torch.all(frac == 1.0 / M) and torch.all(prob == 1.0 / M)


def test_empty_input_and_out_of_range_groups():
    M = 4
    loss, frac, prob = mg.moga_balance_loss(torch.empty(0, dtype=torch.int32).cuda(), torch.empty(0).cuda(), M, ALPHA)
    assert float(loss.item()) == 0.0 and torch.all(frac == 0) and torch.all(prob == 0)
    group = torch.tensor([0, 1, 7, -1, 1, 3], dtype=torch.int32)
    gate = torch.tensor([0.5, 0.25, 0.9, 0.9, 0.75, 1.0])
    loss, frac, prob = mg.moga_balance_loss(group.cuda(), gate.cuda(), M, ALPHA)
    np.testing.assert_allclose(P.to64(frac), np.array([1, 2, 0, 1]) / 6.0, rtol=1e-7)
    np.testing.assert_allclose(P.to64(prob), np.array([0.5, 1.0, 0.0, 1.0]) / 6.0, rtol=1e-7)


@pytest.mark.parametrize("N,M", [(4096, 8), (100001, 32), (3, 256)])
def test_balance_loss_gradient_matches_oracle(N, M):
    group, gate = case(N, M, seed=N + M + 1, skew=True)
    ref = orc.balance_loss_bwd(group.numpy(), M, ALPHA)
    _, frac, _ = mg.moga_balance_loss(group.cuda(), gate.cuda(), M, ALPHA)
    fresh = mg.moga_balance_loss_bwd(group.cuda(), frac, ALPHA)
    np.testing.assert_allclose(P.to64(fresh), ref, rtol=2e-6, atol=0)
    base = torch.randn(N, generator=torch.Generator().manual_seed(5))
    acc = base.clone().cuda()
    mg.moga_balance_loss_bwd(group.cuda(), frac, ALPHA, d_loss=-2.5, d_gate=acc)
    np.testing.assert_allclose(P.to64(acc), P.to64(base) - 2.5 * ref, rtol=1e-6, atol=1e-9)
    # the upstream gradient as a device scalar (what an autograd caller holds): same result, no host sync
    acc2 = base.clone().cuda()
    mg.moga_balance_loss_bwd(group.cuda(), frac, ALPHA, d_loss=torch.tensor(-2.5, device="cuda"), d_gate=acc2)
    np.testing.assert_allclose(P.to64(acc2), P.to64(base) - 2.5 * ref, rtol=1e-6, atol=1e-9)


def test_router_gradient_of_attention_plus_balancing_loss():
    """Loss = sum(O * dO) + L_balance on C1 shapes: the gate gradient of the balancing term is added
    before the router backward; dW against the oracle's router backward of the summed gate gradient."""
    w = wl.WORKLOADS["C1b"]
    inp = wl.make_inputs(w, "cpu")
    X, W, Q, K, V, dO = (P.to64(inp[k]) for k in ("X", "W", "Q", "K", "V", "dO"))
    f = orc.moga_forward(X, W, Q, K, V, w.scale)
    b = orc.moga_backward(f, X, W, dO, w.scale)
    d_gate_total = b["d_gate"] + orc.balance_loss_bwd(f["group"], w.M, ALPHA)
    dW, _, _ = orc.route_bwd(X, W, f["probs"], f["group"], f["gate"], d_gate_total)
    d = {k: inp[k].cuda() for k in ("X", "W", "Q", "K", "V", "dO")}
    fg = mg.moga_forward(d["X"], d["W"], d["Q"], d["K"], d["V"], w.scale)
    assert not P.check_assignment(fg["group"].cpu().numpy(), f)
    d_oh, d_gate = mg.moga_unpermute_bwd(d["dO"], fg["oh"], fg["perm"], fg["gate"])
    loss, frac, _ = mg.moga_balance_loss(fg["group"], fg["gate"], w.M, ALPHA)
    mg.moga_balance_loss_bwd(fg["group"], frac, ALPHA, d_gate=d_gate)
    d_w, _ = mg.moga_route_bwd(d["X"], d["W"], fg["probs"], fg["group"], fg["gate"], d_gate)
    torch.cuda.synchronize()
    np.testing.assert_allclose(float(loss.item()), orc.balance_loss(f["group"], f["gate"], w.M, ALPHA)[0], rtol=1e-5)
    e = P.assert_close_f32(P.to64(d_w), dW, "dW with balancing term")
    say(f"  dW rel err {e:.3e}; balancing share of |d_gate|: "
        f"{np.abs(d_gate_total - b['d_gate']).max() / np.abs(b['d_gate']).max():.2e}")
