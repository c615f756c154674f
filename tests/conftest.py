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


@pytest.fixture(params=["auto", "2wg"])
def kernel_variant(request, monkeypatch):
    """Runs a GPU test once per schedule of the forward: the library's own choice (the interleaved
    kernel) and the two-workgroup kernel forced wherever it applies (calls it does not cover take
    the library's choice)."""
    import paper_2603_05503_amd as pkg
    from paper_2603_05503_amd import binding

    if request.param == "auto":
        return request.param
    plain = binding.sparse_attn_fwd
    forced = binding.KERNEL_TWO_WORKGROUPS

    def variant(q, k, v, out, pattern, scale, *args, **kwargs):
        if "kernel" in kwargs:
            return plain(q, k, v, out, pattern, scale, *args, **kwargs)
        try:
            return plain(q, k, v, out, pattern, scale, *args, kernel=forced, **kwargs)
        except binding.CalibattError as e:
            if e.status != -3:  # CALIBATT_ERR_UNSUPPORTED: the forced kernel does not cover this call
                raise
            return plain(q, k, v, out, pattern, scale, *args, **kwargs)

    monkeypatch.setattr(pkg, "sparse_attn_fwd", variant)
    monkeypatch.setattr(binding, "sparse_attn_fwd", variant)
    return request.param
