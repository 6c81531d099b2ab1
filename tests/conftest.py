import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def sa():
    """The GPU library's Python binding; GPU tests fail loudly when it cannot load."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2306_06446_amd as pkg
    pkg.load_library()
    return pkg
