import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def lib():
    """The ctypes binding with the built HIP library loaded (GPU tests)."""
    import paper_2603_05503_amd as pkg

    return pkg


@pytest.fixture(params=["2wg", "pipe", "pp"])
def kernel_variant(request, monkeypatch):
    """Runs a GPU test once per kernel: the library reads CALIBATT_KERNEL on every call.  "pipe"
    selects the in-wave pipelined kernel for 128 x 128 x 128 blocks, "pp" the ping-pong kernel for
    shapes with block_q <= block_k; shapes a variant does not cover take the default
    two-workgroup kernel."""
    monkeypatch.setenv("CALIBATT_KERNEL", request.param)
    return request.param
