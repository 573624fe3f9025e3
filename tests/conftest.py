import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def spd():
    """The ctypes binding of the HIP library (built in-tree if it is not there yet)."""
    from paper_2502_20727_amd import binding
    return binding


@pytest.fixture(scope="session")
def gpu(spd):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this process")
    torch.cuda.set_device(0)
    return torch.device("cuda:0")
