"""The whole path can be recorded into a HIP graph and replayed: every C-ABI call only enqueues
kernels on the given stream (no host synchronisation, no memset nodes).  Each replay is checked
against the eager result, with eager work and synchronisations between the replays."""
import pytest
import torch

from paper_2510_18692_amd import binding as mg
from paper_2510_18692_amd import workloads as wl

pytestmark = pytest.mark.gpu

KEYS_F = ("group", "gate", "counts", "cu_seqlens", "perm", "oh", "lse", "o")
KEYS_B = ("d_q", "d_k", "d_v", "d_w", "d_gate")


@pytest.mark.parametrize("name,N", [("C1b", 4096), ("C5", 3 * 1560)])
def test_forward_backward_in_a_graph_matches_eager_on_every_replay(name, N):
    w = wl.scaled(wl.WORKLOADS[name], N=N)
    inp = wl.make_inputs(w, "cuda")
    args = (inp["X"], inp["W"], inp["Q"], inp["K"], inp["V"], w.scale)

    def run():
        f = mg.moga_forward(*args)
        loss, frac, prob = mg.moga_balance_loss(f["group"], f["gate"], w.M, 0.1)
        b = mg.moga_backward(f, inp["X"], inp["W"], inp["dO"], w.scale)
        return f, b, loss

    f0, b0, l0 = run()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):      # warm-up on the capture stream, as torch asks
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fg, bg, lg = run()
    for rep in range(3):
        print(f"replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        for k in KEYS_F:
            assert torch.equal(fg[k], f0[k]), (rep, k)
        for k in KEYS_B:
            assert torch.equal(bg[k], b0[k]), (rep, k)
        assert torch.equal(lg, l0)
        fe, be, _ = run()              # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(fe["o"], f0["o"]) and torch.equal(be["d_w"], b0["d_w"])
