"""The bf16 attention calls choose between two sets of kernels from the mean group size (8-wave blocks
with 256 / 128-row tiles, or 4-wave blocks with tiles half as large for small groups).  The shape cases
of the other GPU tests are small, so by default they all land on the small-group set: here the same
cases (tile edges, empty groups, separate query and key lists) run with each set forced in turn, each
against the oracle."""
import pytest

from paper_2510_18692_amd import binding as mg
from tests import test_gpu_backward as tb
from tests import test_gpu_forward as tf
from tests import test_gpu_varlen as tv

pytestmark = pytest.mark.gpu

SHAPES = [
    ([300, 0, 1, 129, 257, 64, 2, 511], 3),
    ([4095, 4096, 17], 2),
    ([40], 1),
    ([288, 289, 319, 320, 321, 352, 575, 576, 577, 33, 32, 31, 63, 64, 65, 95, 96, 97, 127, 128, 129, 255, 256, 257, 1, 2], 1),
]


@pytest.fixture(params=[0, 1 << 40], ids=["large-group kernels", "small-group kernels"])
def kernel_set(request):
    mg.set_small_group_rows(request.param)
    yield request.param
    mg.set_small_group_rows(-1)


@pytest.mark.parametrize("sizes,H", SHAPES)
def test_forward_with_each_kernel_set(kernel_set, sizes, H):
    tf.test_group_attention_forward_matches_oracle(sizes, H, 128, "bf16")


@pytest.mark.parametrize("sizes,H", SHAPES)
def test_backward_with_each_kernel_set(kernel_set, sizes, H):
    tb.test_group_attention_backward_matches_oracle(sizes, H, 128, "bf16")


def test_peaked_rows_with_each_kernel_set(kernel_set):
    tf.test_group_attention_bf16_peaked_rows_have_teeth()


def test_separate_query_and_key_lists_with_each_kernel_set(kernel_set):
    tv.run_case([100, 0, 257, 64, 1, 300], [164, 10, 257, 0, 40, 900], 2, 128, "bf16", seed=3)
    tv.run_case([1300, 70], [1560, 2000], 1, 128, "bf16", seed=4)
