import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU harness)")


@pytest.fixture(scope="session")
def blas():
    """The ctypes binding of libmxblas.so (fails loudly if the library is not built)."""
    from paper_2411_07211_amd import blas as b
    return b


@pytest.fixture(scope="session")
def ctx(blas):
    """A handle with a workspace, on torch's current stream of cuda:0."""
    import torch
    assert torch.cuda.is_available(), "gpu-marked test run without a GPU"
    return blas.Context(device="cuda:0")
