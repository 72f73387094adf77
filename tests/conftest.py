import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def hip_device():
    """torch device for GPU tests; the tests are marked gpu, so this only runs on the GPU machine."""
    import torch
    assert torch.cuda.is_available(), "GPU test started without a GPU"
    return torch.device("cuda:0")
