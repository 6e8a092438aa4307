"""Host-side checks of the measurement helpers: the bench-only library exports its microbenchmarks and
refuses bad arguments without a GPU; the power sampler and the traffic reader degrade to "no data"."""
import ctypes
import os

from paper_2510_18692_amd import build, profiling


def test_bench_library_exports_and_validates():
    assert os.path.exists(build.BENCH_LIB)
    lib = ctypes.CDLL(build.BENCH_LIB)
    for name in ("moga_bench_mfma_loop", "moga_bench_copy", "moga_bench_mix_loop"):
        assert hasattr(lib, name), name
    lib.moga_bench_mfma_loop.restype = ctypes.c_double
    lib.moga_bench_mfma_loop.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.moga_bench_mfma_loop(0, 10, None, None) == -1.0
    lib.moga_bench_copy.restype = ctypes.c_double
    lib.moga_bench_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    assert lib.moga_bench_copy(None, None, 16, None) == -1.0
    assert lib.moga_bench_copy(ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000), 24, None) == -1.0   # not a multiple of 16
    lib.moga_bench_mix_loop.restype = ctypes.c_double
    lib.moga_bench_mix_loop.argtypes = [ctypes.c_int] * 6 + [ctypes.c_void_p, ctypes.c_void_p]
    assert lib.moga_bench_mix_loop(0, 0, 0, 256, 10, 0, None, None) == -1.0            # no sink
    assert lib.moga_bench_mix_loop(0, 0, 0, 0, 10, 0, ctypes.c_void_p(0x1000), None) == -1.0


def test_the_library_proper_does_not_export_the_microbenchmarks():
    lib = ctypes.CDLL(build.LIB)
    assert not hasattr(lib, "moga_bench_mfma_loop")
    assert not hasattr(lib, "moga_bench_mix_loop")


def test_energy_variants_are_the_ones_the_library_builds():
    src = open(os.path.join(build.CSRC, "bench_peaks.hip")).read()
    for nl, nf, ne in profiling._ENERGY_VARIANTS:
        assert f"MOGA_MIX({nl}, {nf}, {ne})" in src


def test_power_sampler_without_a_sensor_reports_nothing():
    bp = profiling.BoardPower()
    bp.path = None        # as on a machine without the hwmon file
    with bp:
        pass
    assert bp.summary() is None and bp.cap_w() is None


def test_power_sampler_reads_a_sensor_file(tmp_path):
    (tmp_path / "power1_input").write_text("1234000000\n")
    (tmp_path / "power1_cap").write_text("1400000000\n")
    bp = profiling.BoardPower(period_s=0.001, settle_s=0.0)
    bp.path = str(tmp_path / "power1_input")
    with bp:
        import time
        time.sleep(0.02)
    s = bp.summary()
    assert s["mean_w"] == 1234.0 and s["max_w"] == 1234.0 and s["cap_w"] == 1400.0 and s["samples"] >= 2


def test_traffic_reader_returns_bytes_per_call_for_the_profiled_workload():
    t = profiling.read_call_traffic("C4b")
    assert t["moga_group_attn_bwd"] > 1e10 and t["moga_group_attn_fwd"] > 1e10
    assert profiling.read_call_traffic("no-such-workload") == {}
