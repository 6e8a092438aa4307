"""The host-side builder of the static group lists (Section 3.2) against the oracle's lists.
Runs without a GPU: the builder is plain host code inside the C-ABI library."""
import numpy as np
import pytest

from oracle import stga_oracle as sto
from paper_2510_18692_amd import binding as mg

CASES = [
    (6, 4, 4, 2, 2, 2, [0, 0, 0, 1, 1, 1], 1, 1),
    (7, 3, 5, 2, 3, 3, [0, 0, 1, 1, 1, 1, 2], 1, 1),
    (4, 2, 2, 2, 2, 4, [0, 0, 0, 0], 1, 1),
    (5, 4, 2, 4, 1, 1, [3, 3, 5, 5, 9], 1, 1),
    (9, 5, 7, 2, 4, 2, [0, 0, 0, 0, 1, 1, 1, 2, 2], 2, 1),
    (12, 6, 8, 3, 4, 3, [0] * 5 + [1] * 7, 0, 2),
    (3, 1, 1, 1, 1, 1, [0, 1, 2], 1, 1),
]


@pytest.mark.parametrize("T,Hh,Ww,wh,ww,tg,shot,ap,an", CASES)
def test_builder_equals_oracle_lists(T, Hh, Ww, wh, ww, tg, shot, ap, an):
    ref = sto.stga_index(T, Hh, Ww, wh, ww, tg, shot, ap, an)
    got = mg.moga_stga_build_index(T, Hh, Ww, wh, ww, tg, shot, ap, an, device=None)
    assert got["n_groups"] == ref["n_groups"] and got["n_keys"] == len(ref["kv_index"])
    for k in ("q_index", "cu_q", "kv_index", "cu_k"):
        assert np.array_equal(got[k], ref[k]), k
    N = T * Hh * Ww
    assert np.array_equal(got["q_slot"][got["q_index"]], np.arange(N))
    # inverse lists: every slot once, ascending per token, pointing back at the token
    assert got["inv_cu"][0] == 0 and got["inv_cu"][-1] == got["n_keys"]
    assert sorted(got["inv_slots"].tolist()) == list(range(got["n_keys"]))
    for t in range(N):
        sl = got["inv_slots"][got["inv_cu"][t]:got["inv_cu"][t + 1]]
        assert np.all(np.diff(sl) > 0) and np.all(got["kv_index"][sl] == t)


def test_builder_rejects_bad_arguments():
    lib = mg.load()
    import ctypes
    shots = np.array([0, 1, 0], dtype=np.int32)     # not non-decreasing
    G, Nk = ctypes.c_int64(), ctypes.c_int64()
    sp = shots.ctypes.data_as(ctypes.c_void_p)
    assert lib.moga_stga_index_sizes(3, 2, 2, 1, 1, 1, sp, 1, 1, ctypes.byref(G), ctypes.byref(Nk)) == -1
    assert lib.moga_stga_index_sizes(3, 2, 2, 0, 1, 1, sp, 1, 1, ctypes.byref(G), ctypes.byref(Nk)) == -1
    assert lib.moga_stga_index_sizes(3, 2, 2, 1, 1, 1, None, 1, 1, ctypes.byref(G), ctypes.byref(Nk)) == -1


def test_paper_scale_geometry_counts():
    """480p latent grid of the paper (30 x 52 tokens per frame), 372 frames in 12 shots of 31."""
    T, Hh, Ww = 372, 30, 52
    shots = np.repeat(np.arange(12), 31)
    got = mg.moga_stga_build_index(T, Hh, Ww, 6, 13, 4, shots, device=None)
    runs = 12 * 8                                    # 31 frames = 7 runs of 4 + 1 run of 3
    assert got["n_groups"] == runs * 5 * 4
    assert got["cu_q"][-1] == T * Hh * Ww
    per_window = 6 * 13
    expect_keys = T * Hh * Ww + (10 * 2 + 2 * 1) * 8 * 20 * per_window   # interior shots add 2 frames per run
    assert got["n_keys"] == expect_keys
