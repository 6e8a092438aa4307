"""Turns rocprofv3 output of `bench.py` runs into the short text summaries kept under profiles/,
and reads the per-call HBM traffic back for bench.py's `roofline.traffic`.

Usage (after the rocprofv3 runs named in each summary have written their CSV files):

    python -m paper_2510_18692_amd.profiling layer    --workload C4b --stats S_kernel_stats.csv \\
        --fetch F_counter_collection.csv --write W_counter_collection.csv --bench-log run.log --out-dir profiles
    python -m paper_2510_18692_amd.profiling counters --workload C4b --stats S_kernel_stats.csv \\
        --csv pass1_counter_collection.csv pass2_counter_collection.csv --out profiles/attn_C4b_mfma_counters.md

    python -m paper_2510_18692_amd.profiling energy --out profiles/mfma_energy_probe.md     (runs on the GPU)

Only `energy` needs a GPU; nothing here is imported by the library's hot path.  `BoardPower` samples the
board power sensor (hwmon, read-only) for bench.py and for `energy`.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import glob
import os
import re
import threading
import time

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


class BoardPower:
    """Samples the GPU board power (hwmon `power1_input`, microwatts, of the first card that has one) from a
    thread while a `with` block runs.  `summary()` is None where the sensor cannot be read.  The sensor
    averages over some tens of milliseconds, so the mean skips the first `settle_s` seconds."""

    def __init__(self, period_s=0.01, settle_s=0.15):
        files = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self.path = files[0] if files else None
        self.period_s, self.settle_s = period_s, settle_s
        self.samples = []   # (seconds since start, watts)
        self._stop = threading.Event()
        self._thread = None

    def _read(self, path):
        try:
            with open(path) as f:
                return int(f.read().strip()) / 1e6
        except (OSError, ValueError):
            return None

    def _run(self):
        t0 = time.perf_counter()
        while not self._stop.is_set():
            w = self._read(self.path)
            if w is not None:
                self.samples.append((time.perf_counter() - t0, w))
            time.sleep(self.period_s)

    def __enter__(self):
        self.samples = []
        self._stop.clear()
        if self.path:
            self._thread = threading.Thread(target=self._run, daemon=True)
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        if self._thread:
            self._thread.join()
        return False

    def cap_w(self):
        return self._read(os.path.join(os.path.dirname(self.path), "power1_cap")) if self.path else None

    def summary(self):
        late = [w for t, w in self.samples if t >= self.settle_s] or [w for _, w in self.samples]
        if not late:
            return None
        cap = self.cap_w()
        return {"mean_w": round(sum(late) / len(late), 1), "max_w": round(max(late), 1), "cap_w": cap,
                "samples": len(late), "source": "hwmon power1_input, 10 ms period, first 0.15 s skipped"}


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


def _watts(line):
    bp = line.get("roofline", {}).get("board_power")
    return f"{bp['mean_w']:.0f} W mean, {bp['max_w']:.0f} W max (cap {bp['cap_w']:.0f} W)" if bp else "not readable"


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
    rocprofv3 --pmc GRBM_GUI_ACTIVE SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES --kernel-trace -d gpurun_out/pmc_zero -o zero --output-format csv -- python3 bench.py --workload {args.workload} --steps 2 --warmup 1 --values zeros --no-cpu-baseline
    python -m paper_2510_18692_amd.profiling power ...   (writes this file)

| kernel | random: ms | clock GHz | MFMA busy | zeros: ms | clock GHz | MFMA busy | time ratio |
|---|---|---|---|---|---|---|---|
""" + "\n".join(rows) + f"""

Whole step: {lr['ms_per_step']} ms ({lr['value']} effective TFLOP/s) on random data, {lz['ms_per_step']} ms ({lz['value']}) on zeros.
Measured peaks of the random run (register-resident MFMA loop on random operands, plain copy): {json.dumps(pk)}.
Board power over the timed steps (hwmon sensor, `roofline.board_power` of the two bench lines): random {_watts(lr)}, zeros {_watts(lz)}.

MFMA busy (cycles the matrix pipes are occupied / SIMD cycles) is a property of the instruction stream and is the
same in both runs; what changes is the clock the power management grants.  On random data the kernels are held at
1.7-2.0 GHz of the 2.4 GHz the chip reaches on zeros, and a loop of nothing but MFMAs on random operands is held
at the rate reported above: that rate, not 2.5 PFLOP/s, is what bf16 matrix work can reach on this chip.
"""
    open(args.out, "w").write(txt)
    print(txt)


# (LDS fragment reads, fmas, exp2s) per MFMA: the combinations libmoga_bench.so builds
_ENERGY_VARIANTS = [(0, 0, 0), (1, 0, 0), (2, 0, 0), (0, 2, 0), (0, 4, 0), (0, 6, 0), (0, 0, 1), (0, 0, 2), (1, 4, 1)]


def write_energy(args):
    """Runs the mixed MFMA loop of libmoga_bench.so at the board's power limit and prices an LDS fragment
    read, an fma and an exp2 in units of the energy of one MFMA."""
    import ctypes

    import torch

    from . import build as _build
    lib = ctypes.CDLL(_build.BENCH_LIB)
    fn = lib.moga_bench_mix_loop
    fn.restype = ctypes.c_double
    fn.argtypes = [ctypes.c_int] * 6 + [ctypes.c_void_p, ctypes.c_void_p]
    blocks, iters, reps = 256, args.iters, args.reps
    with BoardPower(settle_s=0.0) as bp:   # before the first launch: the idle board
        time.sleep(0.3)
    idle = (bp.summary() or {}).get("mean_w")
    cap = bp.cap_w()
    sink = torch.empty(blocks * 512, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    res = {}
    for zero in (0, 1):
        for nl, nf, ne in _ENERGY_VARIANTS:
            assert fn(nl, nf, ne, blocks, 2000, zero, sink.data_ptr(), st) > 0
            torch.cuda.synchronize()
            with BoardPower() as bp:
                e0.record()
                flop = sum(fn(nl, nf, ne, blocks, iters, zero, sink.data_ptr(), st) for _ in range(reps))
                e1.record()
                torch.cuda.synchronize()
            sec = e0.elapsed_time(e1) * 1e-3
            pw = bp.summary()
            res[(zero, nl, nf, ne)] = {"tflops": flop / sec / 1e12, "sec": sec, "watts": pw["mean_w"] if pw else None,
                                       "busy_ghz": flop / 32768.0 * 32.0 / 1024.0 / sec / 1e9}
            print(f"zero={zero} lds={nl} fma={nf} exp={ne}: {res[(zero, nl, nf, ne)]}", flush=True)

    def jpf(r):   # joules per PFLOP of MFMA work
        return r["watts"] / r["tflops"] * 1e3 if r["watts"] else float("nan")

    rows = []
    for zero in (0, 1):
        for nl, nf, ne in _ENERGY_VARIANTS:
            r = res[(zero, nl, nf, ne)]
            rows.append(f"| {'zeros' if zero else 'random'} | {nl} | {nf} | {ne} | {r['tflops']:.0f} | {r['busy_ghz']:.2f} | "
                        f"{r['watts'] if r['watts'] is not None else 'n/a'} | {jpf(r):.0f} |")
    base = res[(0, 0, 0, 0)]

    def per_unit(key, n):
        return (jpf(res[key]) - jpf(base)) / n

    lds1 = per_unit((0, 1, 0, 0), 1)
    fma1 = per_unit((0, 0, 6, 0), 6)
    exp1 = per_unit((0, 0, 0, 2), 2)
    txt = f"""# What an MFMA, an LDS fragment read, an fma and an exp2 cost at the board's power limit

Command (from the repository root on one MI355X):

    python -m paper_2510_18692_amd.profiling energy --out profiles/mfma_energy_probe.md

`moga_bench_mix_loop` (libmoga_bench.so): 256 blocks of 8 waves (two per SIMD), {reps} launches of {iters} iterations of
8 register-resident 32x32x16 bf16 MFMAs per wave; per MFMA the stated number of 1 KB LDS fragment reads (16 bytes per
lane, conflict-free, the fragment is the A or B operand six MFMAs later), fp32 fmas and exp2s.  Power: hwmon
`power1_input` sampled every 10 ms during the launches (cap {cap} W, idle {idle} W).  "busy x GHz" = MFMA pipe cycles
per SIMD per nanosecond (2.4 = every cycle of the top clock).  J/PFLOP = board power / MFMA rate.

| operands | LDS reads / MFMA | fma / MFMA | exp2 / MFMA | MFMA TFLOP/s | busy x GHz | board W | J/PFLOP |
|---|---|---|---|---|---|---|---|
""" + "\n".join(rows) + f"""

On random operands every variant sits at the same board power: the power management trades clock for switching
activity, so the rate is set by the energy per MFMA and its companions.  Differences against the plain loop
({jpf(base):.0f} J/PFLOP): one 1 KB LDS fragment read per MFMA costs {lds1:.0f} J/PFLOP ({100 * lds1 / jpf(base):.0f} % of an MFMA), one fma
{fma1:.0f} ({100 * fma1 / jpf(base):.1f} %), one exp2 {exp1:.0f} ({100 * exp1 / jpf(base):.1f} %).  The attention kernels read one 1 KB fragment per MFMA
(32 rows per wave), evaluate about one exp2 and three to four other vector instructions per MFMA and keep the matrix
pipes busy 57-69 % of the cycles; the sum of those prices plus the idle power over the longer run time is what separates
their 1.15-1.3 PFLOP/s of executed MFMA work from the plain loop's rate.
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
    g = sub.add_parser("energy")
    g.add_argument("--iters", type=int, default=400000)
    g.add_argument("--reps", type=int, default=8)
    g.add_argument("--out", required=True)
    g.set_defaults(fn=write_energy)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
