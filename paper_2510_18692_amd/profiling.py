"""Turns rocprofv3 output of `bench.py` runs into the short text summaries kept under profiles/,
and reads the per-call HBM traffic back for bench.py's `roofline.traffic`.

Usage (after the rocprofv3 runs named in each summary have written their CSV files):

    python -m paper_2510_18692_amd.profiling layer    --workload C4b --stats S_kernel_stats.csv \\
        --fetch F_counter_collection.csv --write W_counter_collection.csv --bench-log run.log --out-dir profiles
    python -m paper_2510_18692_amd.profiling counters --workload C4b --stats S_kernel_stats.csv \\
        --csv pass1_counter_collection.csv pass2_counter_collection.csv --out profiles/attn_C4b_mfma_counters.md

No GPU is needed for either; nothing here is imported by the library's hot path.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# kernel name fragment -> C-ABI call it belongs to (scatter_rows serves two calls: see _call_of)
_KERNEL_CALL = [
    ("route_mfma", "moga_route"), ("route_generic", "moga_route"),
    ("chunk_hist", "moga_permute"), ("chunk_scan", "moga_permute"), ("chunk_rank", "moga_permute"),
    ("gather_rows_kernel", "moga_permute"),
    ("attn_fwd", "moga_group_attn_fwd"),
    ("unpermute_bwd", "moga_unpermute_bwd"),
    ("attn_bwd", "moga_group_attn_bwd"),
    ("route_bwd", "moga_route_bwd"),
]


def short_name(kernel: str) -> str:
    return kernel.split("(")[0].replace("void ", "").strip()


def read_kernel_stats(path):
    """rocprofv3 --stats kernel summary -> {kernel: dict(calls, avg_ms, total_ms, pct)}"""
    out = {}
    for r in csv.DictReader(open(path)):
        out[short_name(r["Name"])] = {"calls": int(r["Calls"]), "avg_ms": float(r["AverageNs"]) / 1e6,
                                      "total_ms": float(r["TotalDurationNs"]) / 1e6, "pct": float(r["Percentage"])}
    return out


def read_counters(path):
    """rocprofv3 --pmc counter_collection.csv -> {kernel: {counter: [value per dispatch, in dispatch order]}}"""
    rows = list(csv.DictReader(open(path)))
    rows.sort(key=lambda r: int(r.get("Dispatch_Id", 0)))
    out = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in rows:
        out[short_name(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return out


def _call_of(kernel: str, nth_dispatch: int):
    if "scatter_rows_kernel" in kernel:      # first launch of a step: moga_unpermute; second: moga_permute_bwd
        return "moga_unpermute" if nth_dispatch % 2 == 0 else "moga_permute_bwd"
    for frag, call in _KERNEL_CALL:
        if frag in kernel:
            return call
    return None


def _bench_line(path):
    for l in open(path):
        if l.startswith("{"):
            return json.loads(l)
    raise RuntimeError(f"no JSON line in {path}")


def traffic_path(workload: str) -> str:
    return os.path.join(ROOT, "profiles", f"layer_{workload}_hbm_traffic.md")


def read_call_traffic(workload: str):
    """{C-ABI call: HBM bytes per call} from the tracked traffic summary of `workload` ({} if there is none)."""
    path = traffic_path(workload)
    if not os.path.exists(path):
        return {}
    out = {}
    for l in open(path):
        m = re.match(r"\|\s*(moga_[a-z_]+)\s*\|\s*([0-9.]+)\s*GB\s*\|", l)
        if m:
            out[m.group(1)] = float(m.group(2)) * 1e9
    return out


def write_layer(args):
    stats = read_kernel_stats(args.stats)
    F, W = read_counters(args.fetch), read_counters(args.write)
    line = _bench_line(args.bench_log)
    wl = args.workload
    cal_f = [v for k, d in F.items() if "moga_bench::copy_kernel" in k for v in d["FETCH_SIZE"]]
    cal_w = [v for k, d in W.items() if "moga_bench::copy_kernel" in k for v in d["WRITE_SIZE"]]
    gib_kib = float(1 << 20)
    ff = gib_kib / cal_f[0] if cal_f else 2.0
    fw = gib_kib / cal_w[0] if cal_w else 1.0
    per_call = collections.defaultdict(float)
    rows = []
    for k in sorted(F, key=lambda k: -sum(F[k]["FETCH_SIZE"])):
        if "moga::" not in k:
            continue
        fs, ws = F[k]["FETCH_SIZE"], W.get(k, {}).get("WRITE_SIZE", [])
        for i, f in enumerate(fs):
            w_ = ws[i] if i < len(ws) else 0.0
            rd, wr = f * ff * 1024, w_ * fw * 1024
            call = _call_of(k, i)
            if call:
                per_call[call] += (rd + wr) / max(1, len(fs) // (2 if "scatter_rows" in k else 1))
            rows.append(f"| {k} #{i} | {f:,.0f} | {w_:,.0f} | {rd / 1e9:.2f} | {wr / 1e9:.2f} |")
    calls = line.get("calls", {})
    ctab = []
    for c, b in per_call.items():
        ms = calls.get(c, {}).get("ms")
        rate = f"{b / ms / 1e6:.0f} GB/s over {ms:.2f} ms" if ms else "-"
        ctab.append(f"| {c} | {b / 1e9:.2f} GB | {rate} |")
    cmd = ("rocprofv3 --pmc {c} --kernel-trace -d gpurun_out/pmc_{n} -o {n} --output-format csv -- "
           f"python3 bench.py --workload {wl} --steps 1 --warmup 0 --no-cpu-baseline --no-measured-peaks --calibrate-copy")
    txt = f"""# HBM traffic per kernel launch (rocprofv3 PMC), workload {wl}

Commands (one counter per run, from the repository root on one MI355X):

    {cmd.format(c="FETCH_SIZE", n="fetch")}
    {cmd.format(c="WRITE_SIZE", n="write")}
    python -m paper_2510_18692_amd.profiling layer --workload {wl} ...   (writes this file)

Calibration: `--calibrate-copy` runs the library's plain copy kernel on 1 GiB (1,048,576 KiB read, the same written).
For that copy FETCH_SIZE reads {cal_f[0] if cal_f else float('nan'):,.0f} KiB (factor {ff:.2f}) and WRITE_SIZE reads {cal_w[0] if cal_w else float('nan'):,.0f} KiB (factor {fw:.2f}).
Columns: raw counters in KiB per dispatch, then bytes scaled by those factors.  `#i` is the i-th launch of the kernel
in the step (scatter_rows_kernel: #0 is moga_unpermute, #1 is moga_permute_bwd).

| kernel launch | FETCH_SIZE KiB | WRITE_SIZE KiB | HBM read GB | HBM written GB |
|---|---|---|---|---|
""" + "\n".join(rows) + """

Per C-ABI call (bench.py reads this table for `roofline.traffic`; rates use the HIP-event time of the same run):

| call | HBM bytes | rate |
|---|---|---|
""" + "\n".join(ctab) + "\n"
    open(os.path.join(args.out_dir, f"layer_{wl}_hbm_traffic.md"), "w").write(txt)
    krows = [f"| {k} | {v['calls']} | {v['avg_ms']:.3f} | {v['total_ms']:.2f} | {v['pct']:.3f} |"
             for k, v in sorted(stats.items(), key=lambda kv: -kv[1]["total_ms"]) if "moga::" in k]
    clines = "\n".join(f"- {k}: {v['ms']} ms, {v['achieved']} {v['unit']} ({100 * v['frac']:.1f} % of {v['peak']} {v['unit']})"
                       for k, v in calls.items())
    steps = line.get("steps", 0) + line.get("warmup", 0)
    txt = f"""# rocprofv3 kernel stats: whole MoGA layer, workload {wl}

{line['config']['workload']}

Command (run from the repository root on one MI355X):

    rocprofv3 --kernel-trace --stats -d gpurun_out/prof_{wl} -o {wl} --output-format csv -- python3 bench.py --workload {wl} --steps {line.get('steps')} --warmup {line.get('warmup')} --no-cpu-baseline

{steps} launches of every kernel (warm-up and timed steps).  Library kernels only (torch's input-generation kernels omitted):

| kernel | calls | avg ms | total ms | % of GPU time |
|---|---|---|---|---|
""" + "\n".join(krows) + f"""

bench.py line of the same run (HIP-event timing per C-ABI call):

{clines}
- whole step: {line['ms_per_step']} ms, {line['value']} effective TFLOP/s
- measured peaks of the same run: {json.dumps(line.get('roofline', {}).get('measured_peak'))}
"""
    open(os.path.join(args.out_dir, f"layer_{wl}_kernel_stats.md"), "w").write(txt)
    print(txt)


def write_counters(args):
    stats = read_kernel_stats(args.stats) if args.stats else {}
    merged = collections.defaultdict(dict)
    for path in args.csv:
        for k, d in read_counters(path).items():
            for c, vals in d.items():
                merged[k][c] = sum(vals) / len(vals)
    want = [k for k in merged if any(s in k for s in ("attn_fwd_bf16", "attn_bwd_dkdv", "attn_bwd_dq", "route_mfma",
                                                      "route_bwd_dw_mfma"))]
    names = sorted({c for k in want for c in merged[k]})
    short = [k.replace("moga::", "").split("<")[0] for k in want]
    hdr = "| counter | " + " | ".join(short) + " |\n|---|" + "---|" * len(want)
    rows = ["| " + c + " | " + " | ".join(f"{merged[k].get(c, float('nan')):,.0f}" for k in want) + " |" for c in names]
    derived = []
    for k in want:
        m = merged[k]
        parts = []
        cu_cycles = m.get("SQ_BUSY_CU_CYCLES", 0) / 256.0            # the counter sums the 256 CUs
        if cu_cycles and "SQ_VALU_MFMA_BUSY_CYCLES" in m:            # summed over the 1024 SIMDs
            parts.append(f"MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (4 x SQ_BUSY_CU_CYCLES) = {m['SQ_VALU_MFMA_BUSY_CYCLES'] / 1024 / cu_cycles:.3f} of the SIMD cycles")
        if "GRBM_GUI_ACTIVE" in m and k in stats:                     # summed over the 8 XCDs
            parts.append(f"sustained clock = GRBM_GUI_ACTIVE / 8 / kernel time = {m['GRBM_GUI_ACTIVE'] / 8 / (stats[k]['avg_ms'] * 1e-3) / 1e9:.2f} GHz")
        if "SQ_INSTS_VALU_MFMA_MOPS_BF16" in m and k in stats:
            tf = m["SQ_INSTS_VALU_MFMA_MOPS_BF16"] * 512 / (stats[k]["avg_ms"] * 1e-3) / 1e12
            parts.append(f"executed MFMA rate = MOPS x 512 FLOP / kernel time = {tf:.0f} TFLOP/s ({tf / 2500:.3f} of the published peak)")
        if cu_cycles and "SQ_ACTIVE_INST_VALU" in m:                  # in units of 4 cycles, summed over SIMDs
            parts.append(f"vector ALU active = 4 x SQ_ACTIVE_INST_VALU / SIMD cycles = {4 * m['SQ_ACTIVE_INST_VALU'] / 1024 / cu_cycles:.3f}")
        if m.get("SQ_WAVE_CYCLES") and "SQ_WAIT_INST_LDS" in m:
            parts.append(f"waves waiting for LDS = {m['SQ_WAIT_INST_LDS'] / m['SQ_WAVE_CYCLES']:.3f} of wave cycles, for anything = {m.get('SQ_WAIT_INST_ANY', float('nan')) / m['SQ_WAVE_CYCLES']:.3f}")
        if cu_cycles and "SQ_LDS_IDX_ACTIVE" in m:
            parts.append(f"LDS active = SQ_LDS_IDX_ACTIVE / CU cycles = {m['SQ_LDS_IDX_ACTIVE'] / 256 / cu_cycles:.3f}, bank conflicts {m.get('SQ_LDS_BANK_CONFLICT', 0):,.0f} cycles")
        if m.get("SQ_INSTS_MFMA"):
            parts.append(f"per MFMA: {(m.get('SQ_INSTS_VALU', 0) - m['SQ_INSTS_MFMA']) / m['SQ_INSTS_MFMA']:.2f} other vector instructions, {m.get('SQ_INSTS_LDS', 0) / m['SQ_INSTS_MFMA']:.2f} LDS instructions")
        derived.append("- **" + k + "**: " + "; ".join(parts))
    sets = "\n".join(f"    set {i + 1} ({os.path.basename(os.path.dirname(p))}): " + " ".join(sorted(
        {c for d in read_counters(p).values() for c in d})) for i, p in enumerate(args.csv))
    txt = f"""# MFMA and LDS counters of the matrix-core kernels (rocprofv3 PMC), workload {args.workload}

Commands (one run per counter set, each `timeout -s KILL 300 rocprofv3 --pmc <set> --kernel-trace -d gpurun_out/<dir>
-o <name> --output-format csv -- python3 bench.py --workload {args.workload} --steps 1 --warmup 0 --no-cpu-baseline
--no-measured-peaks`):

{sets}

    python -m paper_2510_18692_amd.profiling counters --workload {args.workload} ...   (writes this file)

Kernel times come from the `--kernel-trace --stats` run summarised in layer_{args.workload}_kernel_stats.md.
Counter values are per dispatch, summed over the chip as rocprofv3 reports them (256 CUs, 1024 SIMDs, 8 XCDs).

{hdr}
""" + "\n".join(rows) + "\n\nDerived:\n\n" + "\n".join(derived) + "\n"
    open(args.out, "w").write(txt)
    print(txt)


def write_block(args):
    stats = read_kernel_stats(args.stats)
    line = _bench_line(args.bench_log)
    rows = list(csv.DictReader(open(args.trace)))
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    att = [(short_name(r["Kernel_Name"]), (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6)
           for r in rows if "moga::attn_" in r["Kernel_Name"] and "delta" not in r["Kernel_Name"]]
    per_pass = len(att) // max(1, line.get("steps", 1) + line.get("warmup", 0))
    last = att[-per_pass:]
    krows = [f"| {k} | {v['calls']} | {v['avg_ms']:.3f} | {v['total_ms']:.2f} | {v['pct']:.3f} |"
             for k, v in sorted(stats.items(), key=lambda kv: -kv[1]["total_ms"]) if "moga::" in k]
    txt = f"""# rocprofv3 kernel stats: three-branch attention block (MoGA + spatial-temporal groups + per-frame groups), fwd+bwd

{line['config']['workload']}; (query, key) pairs {line['config']['pairs']}

Command (run from the repository root on one MI355X):

    rocprofv3 --kernel-trace --stats -d gpurun_out/prof_block -o blk --output-format csv -- python3 bench.py --block --steps {line.get('steps')} --warmup {line.get('warmup')}
    python -m paper_2510_18692_amd.profiling block ...   (writes this file)

| kernel | calls | avg ms | total ms | % of GPU time |
|---|---|---|---|---|
""" + "\n".join(krows) + f"""

bench.py line of the same run: {line['ms_per_step']} ms per pass, {line['value']} effective TFLOP/s over all three branches.

Attention kernels of the last pass in launch order (forward: MoGA, spatial-temporal, per-frame; then the backward
of each branch, dK/dV before dQ), ms:

""" + "\n".join(f"- {k}: {ms:.2f}" for k, ms in last) + "\n"
    open(args.out, "w").write(txt)
    print(txt)


def _per_kernel(counter_csv, trace_csv):
    """{kernel: dict(ms, clock_ghz, mfma_busy)} of one PMC run (GRBM_GUI_ACTIVE, SQ_BUSY_CU_CYCLES, SQ_VALU_MFMA_BUSY_CYCLES)."""
    c = read_counters(counter_csv)
    t = collections.defaultdict(list)
    for r in csv.DictReader(open(trace_csv)):
        t[short_name(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6)
    out = {}
    for k, d in c.items():
        if "moga::attn_" not in k or "delta" in k:
            continue
        m = {n: sum(v) / len(v) for n, v in d.items()}
        ms = sum(t[k]) / len(t[k])
        cu = m["SQ_BUSY_CU_CYCLES"] / 256.0
        out[k] = {"ms": ms, "clock": m["GRBM_GUI_ACTIVE"] / 8 / (ms * 1e-3) / 1e9,
                  "busy": m["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024 / cu}
    return out


def write_power(args):
    rnd = _per_kernel(args.random[0], args.random[1])
    zer = _per_kernel(args.zeros[0], args.zeros[1])
    lr, lz = _bench_line(args.random[2]), _bench_line(args.zeros[2])
    rows = [f"| {k} | {rnd[k]['ms']:.1f} | {rnd[k]['clock']:.2f} | {rnd[k]['busy']:.3f} | {zer[k]['ms']:.1f} | "
            f"{zer[k]['clock']:.2f} | {zer[k]['busy']:.3f} | {rnd[k]['ms'] / zer[k]['ms']:.2f} |" for k in rnd if k in zer]
    pk = lr.get("roofline", {}).get("measured_peak")
    txt = f"""# The attention kernels run at the chip's power limit: random against all-zero operands, workload {args.workload}

Commands (from the repository root on one MI355X; the second run clears Q, K, V and dO after they are drawn, so
routing, group sizes, grids and every instruction executed are identical, only the switching activity differs):

    rocprofv3 --pmc GRBM_GUI_ACTIVE SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES --kernel-trace -d gpurun_out/pmc_rand -o rand --output-format csv -- python3 bench.py --workload {args.workload} --steps 2 --warmup 1 --no-cpu-baseline
    rocprofv3 --pmc GRBM_GUI_ACTIVE SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES --kernel-trace -d gpurun_out/pmc_zero -o zero --output-format csv -- python3 bench.py --workload {args.workload} --steps 2 --warmup 1 --values zeros
    python -m paper_2510_18692_amd.profiling power ...   (writes this file)

| kernel | random: ms | clock GHz | MFMA busy | zeros: ms | clock GHz | MFMA busy | time ratio |
|---|---|---|---|---|---|---|---|
""" + "\n".join(rows) + f"""

Whole step: {lr['ms_per_step']} ms ({lr['value']} effective TFLOP/s) on random data, {lz['ms_per_step']} ms ({lz['value']}) on zeros.
Measured peaks of the random run (register-resident MFMA loop on random operands, plain copy): {json.dumps(pk)}.

MFMA busy (cycles the matrix pipes are occupied / SIMD cycles) is a property of the instruction stream and is the
same in both runs; what changes is the clock the power management grants.  On random data the kernels are held at
1.7-2.0 GHz of the 2.4 GHz the chip reaches on zeros, and a loop of nothing but MFMAs on random operands is held
at the rate reported above: that rate, not 2.5 PFLOP/s, is what bf16 matrix work can reach on this chip.
"""
    open(args.out, "w").write(txt)
    print(txt)


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("layer")
    a.add_argument("--workload", default="C4b")
    a.add_argument("--stats", required=True)
    a.add_argument("--fetch", required=True)
    a.add_argument("--write", required=True)
    a.add_argument("--bench-log", required=True)
    a.add_argument("--out-dir", default=os.path.join(ROOT, "profiles"))
    a.set_defaults(fn=write_layer)
    b = sub.add_parser("counters")
    b.add_argument("--workload", default="C4b")
    b.add_argument("--stats")
    b.add_argument("--csv", nargs="+", required=True)
    b.add_argument("--out", required=True)
    b.set_defaults(fn=write_counters)
    c = sub.add_parser("block")
    c.add_argument("--stats", required=True)
    c.add_argument("--trace", required=True)
    c.add_argument("--bench-log", required=True)
    c.add_argument("--out", required=True)
    c.set_defaults(fn=write_block)
    e = sub.add_parser("power")
    e.add_argument("--workload", default="C4b")
    e.add_argument("--random", nargs=3, required=True, metavar=("COUNTERS_CSV", "TRACE_CSV", "BENCH_LOG"))
    e.add_argument("--zeros", nargs=3, required=True, metavar=("COUNTERS_CSV", "TRACE_CSV", "BENCH_LOG"))
    e.add_argument("--out", required=True)
    e.set_defaults(fn=write_power)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
