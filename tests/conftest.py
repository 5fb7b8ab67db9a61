import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def octo():
    """The ctypes binding over the HIP library; GPU tests fail loudly if it cannot load or no GPU is present."""
    import torch
    from paper_2502_01277_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.lib()  # raises if the shared library is missing
    return binding
