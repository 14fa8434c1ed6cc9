import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def gpu_lib():
    """The ctypes binding of the HIP library; fails loudly if it is not built."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2207_04606_amd as sptir
    sptir.load_library()
    return sptir
