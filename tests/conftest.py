import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def harp():
    """The HIP library behind its ctypes binding, on cuda:0.  Fails loudly when it is not built."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a visible MI355X"
    from paper_2509_24859_amd import binding
    return binding
