"""Helpers shared by the GPU parity tests: error measures, tolerances, the argmax-mismatch rule."""
import numpy as np
import torch

from oracle import moga_oracle as orc
from paper_2510_18692_amd import workloads

F32_REL = 1e-4        # fp32 path: max|a-b| / max|b|
BF16_ABS = 2e-2       # bf16 path: max|a-b| on unit-variance inputs
BF16_REL_MAX = 2e-2   # scale-free companions of the bf16 bound
BF16_REL_L2 = 1e-2
MARGIN = 1e-5         # an argmax mismatch is allowed only below this top-2 logit margin


def to64(t):
    return workloads.to_numpy64(t)


def rel_max(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    den = np.abs(b).max()
    return float(np.abs(a - b).max() / den) if den > 0 else float(np.abs(a - b).max())


def rel_l2(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def assert_close_f32(got, ref, what):
    e = rel_max(got, ref)
    assert e <= F32_REL, f"{what}: max|a-b|/max|b| = {e:.3e} > {F32_REL}"
    return e


def assert_close_bf16(got, ref, what, abs_tol=BF16_ABS):
    d = float(np.abs(np.asarray(got, np.float64) - ref).max())
    rm, rl = rel_max(got, ref), rel_l2(got, ref)
    assert d <= abs_tol, f"{what}: max|a-b| = {d:.3e} > {abs_tol}"
    assert rm <= BF16_REL_MAX, f"{what}: max|a-b|/max|b| = {rm:.3e} > {BF16_REL_MAX}"
    assert rl <= BF16_REL_L2, f"{what}: l2 rel = {rl:.3e} > {BF16_REL_L2}"
    return d, rm, rl


def check_assignment(group_gpu, rt):
    """Compare GPU group ids with the oracle's routing `rt`.

    Returns the list of mismatching tokens (index, gpu id, oracle id, margin).  Fails if any
    mismatch has a float64 top-2 logit margin of 1e-5 or more.
    """
    g = np.asarray(group_gpu)
    bad = np.nonzero(g != rt["group"])[0]
    report = []
    for i in bad:
        top2 = np.sort(rt["r64"][i])[-2:]
        margin = float(top2[1] - top2[0]) if len(top2) == 2 else float("inf")
        report.append((int(i), int(g[i]), int(rt["group"][i]), margin))
    if report:
        print(f"argmax mismatches: {len(report)}; margins: {[f'{m[3]:.2e}' for m in report[:20]]}")
    worst = max((m[3] for m in report), default=0.0)
    assert worst < MARGIN, f"argmax mismatch with top-2 margin {worst:.3e} >= {MARGIN}: {report[:5]}"
    return report


def hat(a_nhd):
    """[N, H, D] numpy (sorted order) -> head-major [H, N, D] as the library lays it out."""
    return np.ascontiguousarray(np.transpose(a_nhd, (1, 0, 2)))


def unhat(t_hnd):
    """library [H, N, D] tensor -> float64 numpy [N, H, D]."""
    return np.transpose(to64(t_hnd), (1, 0, 2))


def dev(a, dtype):
    return torch.as_tensor(np.ascontiguousarray(a)).to(dtype).cuda().contiguous()
