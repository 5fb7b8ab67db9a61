import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _library_is_built():
    """The tests load the library that is built in-tree.  It is (re)built here only if it is missing or older than one of
    its sources: a stale library would test yesterday's kernels."""
    from paper_2502_01277_amd import binding, build
    srcs = [os.path.join(build.CSRC, f) for f in os.listdir(build.CSRC) if f.endswith((".hip", ".cpp", ".h"))]
    srcs.append(os.path.join(ROOT, "include", "octo.h"))
    if not os.path.exists(binding.LIB_PATH) or os.path.getmtime(binding.LIB_PATH) < max(os.path.getmtime(f) for f in srcs):
        build.build(verbose=False)


@pytest.fixture(scope="session")
def octo():
    """The ctypes binding over the HIP library; GPU tests fail loudly if it cannot load or no GPU is present."""
    import torch
    from paper_2502_01277_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.lib()  # raises if the shared library is missing
    return binding
