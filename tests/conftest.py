import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def gpu_device():
    """The one GPU of the box; the HIP library must be the thing that runs."""
    import torch
    if not torch.cuda.is_available():
        pytest.fail("a test marked gpu was run on a machine without a GPU")
    return torch.device("cuda:0")
