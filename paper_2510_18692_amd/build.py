"""Build libmoga.so (the C-ABI HIP library) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoga.so")
BENCH_LIB = os.path.join(HERE, "libmoga_bench.so")   # peak microbenchmarks for bench.py only
EXAMPLE = os.path.join(HERE, "c_abi_example")
SOURCES = ["api.hip", "route.hip", "permute.hip", "attn_fwd.hip", "attn_bwd.hip", "balance.hip", "static_index.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=default",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU ops
    "-Wno-unused-command-line-argument", "-Wno-deprecated-volatile",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source and link the shared library.  Always recompiles."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                        if "packed-fp32-ops" not in l and l.strip())
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{out}")
        if verbose and out:
            print(out, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    # the two peak microbenchmarks bench.py reports beside the published peaks (a library of their own)
    r = subprocess.run([hipcc, *FLAGS, *extra_flags, "-shared", os.path.join(CSRC, "bench_peaks.hip"),
                        "-o", BENCH_LIB], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("bench library build failed:\n" + r.stdout + r.stderr)
    # a torch-free client of the C ABI (run by the GPU tests)
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-I", os.path.join(ROOT, "include"),
                        os.path.join(CSRC, "c_abi_example.cpp"), "-L", HERE, "-lmoga", "-Wl,-rpath,$ORIGIN",
                        "-o", EXAMPLE], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("example build failed:\n" + r.stdout + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
