"""The microbenchmarks behind `roofline.measured_peak` and the energy probe run on the GPU and return
plausible rates (a broken bench library would otherwise only show up in the bench line)."""
import ctypes

import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def test_measured_peaks_are_plausible():
    import bench
    pk = bench.measured_peaks(torch)
    assert 500.0 < pk["mfma_bf16_tflops"] < 2600.0, pk     # published dense bf16 peak: 2,500
    assert 1500.0 < pk["hbm_copy_gbs"] < 8100.0, pk        # published HBM peak: 8,000


def test_mixed_loop_runs_every_built_variant_and_rejects_the_rest():
    from paper_2510_18692_amd import build, profiling
    lib = ctypes.CDLL(build.BENCH_LIB)
    fn = lib.moga_bench_mix_loop
    fn.restype = ctypes.c_double
    fn.argtypes = [ctypes.c_int] * 6 + [ctypes.c_void_p, ctypes.c_void_p]
    blocks, iters = 64, 200
    sink = torch.zeros(blocks * 512, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    for zero in (0, 1):
        for nl, nf, ne in profiling._ENERGY_VARIANTS:
            flop = fn(nl, nf, ne, blocks, iters, zero, sink.data_ptr(), st)
            assert flop == blocks * 8.0 * iters * 8 * 32768.0, (nl, nf, ne)
    torch.cuda.synchronize()
    assert fn(3, 0, 0, blocks, iters, 0, sink.data_ptr(), st) == -1.0      # not built
    assert float(sink.abs().max()) == 0.0                                   # the sink is practically never written


def test_board_power_sampler_returns_watts_or_nothing():
    from paper_2510_18692_amd import profiling
    x = torch.randn(4096, 4096, device="cuda")
    with profiling.BoardPower(settle_s=0.0) as bp:
        for _ in range(20):
            x = (x @ x).clamp_(-1, 1)
        torch.cuda.synchronize()
    s = bp.summary()
    assert s is None or (50.0 < s["mean_w"] < 3000.0 and s["samples"] >= 1)
