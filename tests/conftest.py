import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def aq():
    """The ctypes binding over the HIP library; GPU tests fail loudly if it is missing."""
    import torch
    assert torch.cuda.is_available(), "GPU test without a GPU"
    from paper_1910_01055_amd import binding
    binding.load()  # raises if libactorq.so is not built
    return binding
