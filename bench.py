#!/usr/bin/env python3
"""Benchmark of the MoGA hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic video tokens:
route -> permute -> group attention -> unpermute, and (for workloads with backward)
unpermute_bwd -> group attention bwd -> permute_bwd -> route_bwd.  Inputs are resident in
HBM before the timed region.  The default workload is the paper-scale context (N = 580,320
tokens, 40 heads, head_dim 128, d_model 5120, M = 32) forward + backward.

Prints ONE JSON line: whole-job effective TFLOP/s (within-group attention FLOPs only:
4*H*D*sum n_g^2 forward, 10*H*D*sum n_g^2 backward) as `value`, ms per layer as
`ms_per_step`, a `roofline` object for the dominant call, per-call figures in `calls`,
and the CPU oracle timed on a bounded sample in `cpu_baseline`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published

BENCH_LIB = os.path.join(ROOT, "paper_2510_18692_amd", "libmoga_bench.so")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="C4b", help="C1, C1b, C2, C3, C3b, C3u, C4, C4b (default), C5")
    ap.add_argument("--fused", action="store_true",
                    help="use the gather-fused attention calls (no permuted tensors are materialised): permute builds "
                         "the index only, moga_fused_attn_fwd / _bwd replace gather + attention + scatter")
    ap.add_argument("--graph", action="store_true",
                    help="record one step into a HIP graph and time its replays (whole-step time only; for the "
                         "small, launch-bound workloads)")
    ap.add_argument("--block", action="store_true",
                    help="time the whole three-branch attention block (MoGA + spatial-temporal groups + "
                         "per-frame groups, forward+backward) on the workload's latent grid instead of the MoGA layer")
    ap.add_argument("--shots", type=int, default=12, help="--block: number of equal-length shots")
    ap.add_argument("--window", default="8x13x0",
                    help="--block: spatial window rows x cols x frames per run (0 = a whole shot). The default is the "
                         "4 x 4 partition of the 30 x 52 latent frame that the paper pairs with long contexts")
    ap.add_argument("--small-group-rows", type=int, default=-1,
                    help="override the mean group size below which the bf16 attention calls use their small-group "
                         "kernels (0: never; default -1: the library's own thresholds)")
    ap.add_argument("--values", default="random", choices=["random", "zeros"],
                    help="diagnostic: 'zeros' clears Q, K, V and dO after they are drawn (X, hence the routing and the "
                         "group sizes, stay): the same instruction stream with minimal switching activity, which shows "
                         "how far the chip's power limit, and not the kernels' schedule, bounds the run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="skip the two peak microbenchmarks (register-resident MFMA loop, plain 1 GiB copy)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run the plain 1 GiB copy kernel even with --no-measured-peaks (a kernel of known traffic, "
                         "used to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def algorithmic_work(w, counts):
    """Per call: (bound, algorithmic bytes or flops per launch).  Bytes follow the method's own
    data movement: every tensor a call must read or write, once."""
    from paper_2510_18692_amd import flops
    N, H, D, d, M = w.N, w.H, w.D, w.d_model, w.M
    es = 4 if w.dtype == "f32" else 2
    t = N * H * D * es                      # one [N, H, D] tensor
    work = {
        "moga_route": ("hbm", N * d * es + M * d * 4 + 8 * N + (4 * N * M if w.backward else 0)),
        "moga_permute": ("hbm", 6 * t + 4 * N * 2 + 8 * N + 4 * N),
        "moga_group_attn_fwd": ("mfma", flops.group_attn_fwd_flops(counts, H, D)),
        "moga_unpermute": ("hbm", 2 * t + 8 * N),
    }
    if w.backward:
        work.update({
            "moga_unpermute_bwd": ("hbm", 3 * t + 12 * N),
            "moga_group_attn_bwd": ("mfma", flops.group_attn_bwd_flops(counts, H, D)),
            "moga_permute_bwd": ("hbm", 6 * t + 4 * N),
            "moga_route_bwd": ("hbm", N * d * es + 4 * N * M + 16 * N + M * d * 4),
        })
    work["moga_fused_attn_fwd"] = work["moga_group_attn_fwd"]
    if w.backward:
        work["moga_fused_attn_bwd"] = work["moga_group_attn_bwd"]
    return work


def measured_peaks(torch):
    """What this GPU delivers on two microbenchmarks (a second denominator beside the published peaks):
    a register-resident bf16 MFMA loop and a plain 1 GiB copy, each timed with HIP events, best of 3."""
    import ctypes
    lib = ctypes.CDLL(BENCH_LIB)
    lib.moga_bench_mfma_loop.restype = ctypes.c_double
    lib.moga_bench_mfma_loop.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.moga_bench_copy.restype = ctypes.c_double
    lib.moga_bench_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    st = torch.cuda.current_stream().cuda_stream
    blocks = 1024
    sink = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(3)
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def best(fn):
        rates = []
        for _ in range(4):        # the first run warms up
            e0.record()
            amount = fn()
            e1.record()
            torch.cuda.synchronize()
            assert amount > 0
            rates.append(amount / (e0.elapsed_time(e1) * 1e-3))
        return max(rates[1:])

    tf = best(lambda: lib.moga_bench_mfma_loop(blocks, 20000, sink.data_ptr(), st)) / 1e12
    gb = best(lambda: lib.moga_bench_copy(dst.data_ptr(), src.data_ptr(), src.numel(), st)) / 1e9
    del sink, src, dst
    return {"mfma_bf16_tflops": round(tf, 1), "hbm_copy_gbs": round(gb, 1),
            "how": "register-resident 32x32x16 bf16 MFMA loop (1024 blocks x 4 waves); plain 1 GiB copy kernel"}


def cpu_baseline(w, inp, budget_s=20.0):
    """The oracle as it stands, timed on this host on a bounded sample of the SAME workload: routing and
    the permutation index of all tokens, then softmax_attention (+ its backward) on whole (group, head)
    pairs of the workload's own groups, smallest group first, until the time budget is used."""
    import numpy as np
    from oracle import moga_oracle as orc
    from paper_2510_18692_amd import workloads as wl
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    t64 = wl.to_numpy64
    W64 = t64(inp["W"])
    t_route, parts = 0.0, []
    for s in range(0, w.N, 65536):
        x = t64(inp["X"][s:s + 65536])          # copy to the host and widening: not timed
        t0 = time.perf_counter()
        parts.append(orc.route(x, W64)["group"])
        t_route += time.perf_counter() - t0
    group = np.concatenate(parts)
    t0 = time.perf_counter()
    idx = orc.permute_index(group, w.M)
    t_perm = time.perf_counter() - t0
    import torch
    order = sorted((g for g in range(w.M) if idx["counts"][g] > 0), key=lambda g: idx["counts"][g])
    fl, el, done = 0.0, 0.0, []
    for i in range(64):
        g, h = order[i % len(order)], (7 * i) % w.H
        n = int(idx["counts"][g])
        if n > 24000:        # the score matrix is n^2 float64, several of them live at once
            continue
        members = torch.from_numpy(idx["perm"][idx["cu_seqlens"][g]:idx["cu_seqlens"][g + 1]].astype(np.int64)).to(inp["Q"].device)
        q, k, v = (t64(inp[name][members, h]) for name in ("Q", "K", "V"))
        dA = t64(inp["dO"][members, h]) if w.backward else None
        t0 = time.perf_counter()
        orc.softmax_attention(q, k, v, w.scale)
        fl += 4.0 * n * n * w.D
        if w.backward:
            orc.softmax_attention_bwd(q, k, v, dA, w.scale)
            fl += 10.0 * n * n * w.D
        el += time.perf_counter() - t0
        done.append(n)
        if el > budget_s:
            break
    from paper_2510_18692_amd import flops
    counts = idx["counts"].tolist()
    total = flops.group_attn_fwd_flops(counts, w.H, w.D) + (flops.group_attn_bwd_flops(counts, w.H, w.D) if w.backward else 0)
    rate = fl / el if el > 0 else float("nan")
    layer_s = total / rate + t_route + t_perm
    return {
        "value": rate / 1e12, "unit": "TFLOP/s", "cores": int(threads), "host_cores": os.cpu_count(), "kind": "oracle",
        "measured_s": {"route_all_tokens": round(t_route, 2), "permute_index_all_tokens": round(t_perm, 3),
                       "attention_sample": round(el, 2)},
        "extrapolated_layer_s": round(layer_s, 1),
        "sample": (f"float64 numpy oracle on this workload's own tensors: route of all {w.N} tokens {t_route:.1f} s, "
                   f"permute_index {t_perm:.2f} s (both measured in full); softmax_attention"
                   f"{' + softmax_attention_bwd' if w.backward else ''} on {len(done)} whole (group, head) pairs of its own groups "
                   f"(n = {done}), {fl / 1e12:.2f} TFLOP in {el:.1f} s (measured); whole layer "
                   f"({total / 1e12:.0f} TFLOP) by FLOP ratio: {layer_s:.0f} s (extrapolated); "
                   f"{threads} BLAS threads on {os.cpu_count()} host cores"),
    }


def run_block(args):
    """--block: one pass of the three-branch block (Section 3.2) per step, whole-call timing."""
    import numpy as np
    import torch
    from paper_2510_18692_amd import binding as mg
    from paper_2510_18692_amd import flops
    from paper_2510_18692_amd import workloads as wl
    mg.load()
    w = wl.WORKLOADS[args.workload]
    T, Hh, Ww = (int(v) for v in w.grid.split("x"))
    wh, ww, tg = (int(v) for v in args.window.split("x"))
    tg = tg if tg > 0 else T
    shots = np.minimum(np.arange(T) * args.shots // T, args.shots - 1)
    torch.cuda.set_device(0)
    inp = wl.make_inputs(w, "cuda")
    si = mg.moga_stga_build_index(T, Hh, Ww, wh, ww, tg, shots)
    torch.cuda.synchronize()

    def step():
        fwd = mg.visual_forward(inp["X"], inp["W"], inp["Q"], inp["K"], inp["V"], w.scale, (T, Hh, Ww), si)
        counts = fwd["pm"]["counts"]
        bwd = mg.visual_backward(fwd, inp["X"], inp["W"], inp["dO"], w.scale)
        del fwd, bwd
        return counts

    for _ in range(args.warmup):
        step()
        torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        counts = step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    counts = counts.cpu().tolist()
    cu_q, cu_k = si["cu_q"].cpu().numpy().astype(np.int64), si["cu_k"].cpu().numpy().astype(np.int64)
    pairs = {"moga": flops.sum_sq(counts), "stga": int(((cu_q[1:] - cu_q[:-1]) * (cu_k[1:] - cu_k[:-1])).sum()),
             "frame": T * (Hh * Ww) ** 2}
    total = 14.0 * w.H * w.D * sum(pairs.values())      # 4 forward + 10 backward per pair, head and channel
    print(json.dumps({
        "metric": "three-branch attention block effective TFLOP/s (attention FLOPs of all branches, fwd+bwd)",
        "value": round(total / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name} + static branches: grid {w.grid}, {args.shots} shots, window {args.window}, "
                               f"{si['n_groups']} spatial-temporal groups, {si['n_keys']} listed keys",
                   "pairs": pairs, "pairs_over_N2": round(sum(pairs.values()) / float(w.N) ** 2, 5)},
    }), flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus must be 1. The design notes say how the path would shard by head.",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2510_18692_amd import binding as mg
    from paper_2510_18692_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    mg.load()
    if args.small_group_rows >= 0:
        mg.set_small_group_rows(args.small_group_rows)
    if args.block:
        return run_block(args)
    w = wl.WORKLOADS[args.workload]
    torch.cuda.set_device(0)
    inp = wl.make_inputs(w, "cuda")
    X, W, Q, K, V = inp["X"], inp["W"], inp["Q"], inp["K"], inp["V"]
    dO = inp.get("dO")
    if args.values == "zeros":
        for t in (Q, K, V, dO):
            if t is not None:
                t.zero_()
        args.no_cpu_baseline = True
    torch.cuda.synchronize()

    names = ["moga_route", "moga_permute", "moga_group_attn_fwd", "moga_unpermute"]
    if w.backward:
        names += ["moga_unpermute_bwd", "moga_group_attn_bwd", "moga_permute_bwd", "moga_route_bwd"]
    if args.fused:
        if w.dtype != "bf16":
            print("bench.py: --fused needs a bf16 workload", file=sys.stderr)
            sys.exit(2)
        names = ["moga_route", "moga_permute", "moga_fused_attn_fwd"]
        if w.backward:
            names += ["moga_fused_attn_bwd", "moga_route_bwd"]

    def step_fused(events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        group, gate, probs, _ = mg.moga_route(X, W, want_probs=w.backward)
        mark(1)
        pm = mg.moga_permute(group, w.M)
        mark(2)
        o, lse = mg.moga_fused_attn_fwd(Q, K, V, pm["perm"], gate, pm["cu_seqlens"], w.scale)
        mark(3)
        out = {"counts": pm["counts"], "o": o}
        if w.backward:
            d_q, d_k, d_v, d_gate = mg.moga_fused_attn_bwd(dO, Q, K, V, o, lse, pm["perm"], pm["inv_perm"], gate,
                                                           pm["cu_seqlens"], w.scale)
            mark(4)
            d_w, _ = mg.moga_route_bwd(X, W, probs, group, gate, d_gate)
            mark(5)
            out["d_w"] = d_w
        return out

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        group, gate, probs, _ = mg.moga_route(X, W, want_probs=w.backward)
        mark(1)
        pm = mg.moga_permute(group, w.M, Q, K, V)
        mark(2)
        oh, lse = mg.moga_group_attn_fwd(pm["qh"], pm["kh"], pm["vh"], pm["cu_seqlens"], w.scale)
        mark(3)
        o = mg.moga_unpermute(oh, pm["perm"], gate)
        mark(4)
        out = {"counts": pm["counts"], "o": o}
        if w.backward:
            d_oh, d_gate = mg.moga_unpermute_bwd(dO, oh, pm["perm"], gate)
            mark(5)
            d_qh, d_kh, d_vh = mg.moga_group_attn_bwd(d_oh, pm["qh"], pm["kh"], pm["vh"], oh, lse,
                                                      pm["cu_seqlens"], w.scale)
            mark(6)
            d_q, d_k, d_v = mg.moga_permute_bwd(d_qh, d_kh, d_vh, pm["perm"])
            mark(7)
            d_w, _ = mg.moga_route_bwd(X, W, probs, group, gate, d_gate)
            mark(8)
            out["d_w"] = d_w
        return out

    if args.fused:
        step = step_fused
    peaks = None
    if args.calibrate_copy or not args.no_measured_peaks:
        peaks = measured_peaks(torch)   # includes the plain 1 GiB copy (copy_kernel) that calibrates the PMC counters
    for _ in range(args.warmup):
        out = step()
        torch.cuda.synchronize()
        del out
    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            held = step()
        graph.replay()
        torch.cuda.synchronize()
        tg0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - tg0) * 1e3 / args.steps
        del held, graph
    nev = len(names) + 1
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(nev)] for _ in range(args.steps)]
    from paper_2510_18692_amd import profiling
    torch.cuda.synchronize()
    with profiling.BoardPower() as board:   # a thread that reads the board's power sensor every 10 ms
        t0 = time.perf_counter()
        counts = None
        for s in range(args.steps):
            out = step(evs[s])
            counts = out["counts"]
            del out
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    counts = counts.cpu().tolist()
    work = algorithmic_work(w, counts)
    calls = {}
    for i, n in enumerate(names):
        ms = sum(evs[s][i].elapsed_time(evs[s][i + 1]) for s in range(args.steps)) / args.steps
        bound, amount = work[n]
        if bound == "mfma":
            ach, peak, unit = amount / (ms * 1e-3) / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s"
            if w.dtype == "f32":
                peak = 157.3
        else:
            ach, peak, unit = amount / (ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
        calls[n] = {"ms": round(ms, 4), "bound": bound, "achieved": round(ach, 2), "peak": peak,
                    "unit": unit, "frac": round(ach / peak, 4)}
    dominant = max(calls, key=lambda n: calls[n]["ms"])
    roof = {k: calls[dominant][k] for k in ("bound", "achieved", "peak", "unit", "frac")}
    roof["kernel"] = dominant
    roof["ms"] = calls[dominant]["ms"]
    # HBM bytes of that call from the tracked rocprofv3 summary of this workload (null if there is none)
    roof["traffic"] = profiling.read_call_traffic(w.name).get(dominant)
    # board power over the timed steps (null where the sensor is not readable): the attention calls run at the cap
    roof["board_power"] = board.summary()
    if peaks is not None:
        roof["measured_peak"] = peaks
        den = peaks["mfma_bf16_tflops"] if roof["bound"] == "mfma" else peaks["hbm_copy_gbs"]
        roof["frac_of_measured_peak"] = round(roof["achieved"] / den, 4)

    from paper_2510_18692_amd import flops
    total_flops = flops.group_attn_fwd_flops(counts, w.H, w.D)
    if w.backward:
        total_flops += flops.group_attn_bwd_flops(counts, w.H, w.D)
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    line = {
        "metric": "MoGA layer effective TFLOP/s (within-group attention FLOPs, "
                  + ("fwd+bwd" if w.backward else "fwd") + "); ms/layer in ms_per_step",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic" + (" (Q, K, V, dO cleared: power diagnostic)" if args.values == "zeros" else ""),
        "config": {"workload": f"{w.name}: N={w.N} ({w.grid} latent grid), H={w.H}, D={w.D}, "
                               f"d_model={w.d_model}, M={w.M}, {w.hidden} hidden states, "
                               + ("forward+backward" if w.backward else "forward")
                               + (", gather-fused attention calls" if args.fused else ""),
                   "group_sizes": {"min": min(counts), "max": max(counts),
                                   "sum_sq_over_N2": round(flops.sum_sq(counts) / float(w.N) ** 2, 5)}},
        "roofline": roof,
        "calls": calls,
    }
    if graph_ms is not None:
        line["graph_replay_ms_per_step"] = round(graph_ms, 4)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, inp)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
