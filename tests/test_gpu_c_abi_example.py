"""A client that uses the C ABI without torch (hipMalloc'd buffers only) runs the forward path."""
import os
import subprocess

import pytest

from paper_2510_18692_amd import build as _build

pytestmark = pytest.mark.gpu


def test_torch_free_client_of_the_c_abi():
    if not os.path.exists(_build.EXAMPLE):
        pytest.skip("example not built")
    r = subprocess.run([_build.EXAMPLE], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0 and "C ABI example OK" in r.stdout
