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
    """The GPU library's Python binding; GPU tests fail loudly if it is not built."""
    import torch
    assert torch.cuda.is_available(), "gpu-marked test run without a GPU"
    import paper_2504_17307_amd as pkg
    pkg.load()
    return pkg
