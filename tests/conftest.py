import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


@pytest.fixture(scope="session")
def gpu():
    """The GPU tests must run the HIP library: no fallback, fail loudly."""
    import torch
    assert torch.cuda.is_available(), "GPU test selected but no GPU is visible"
    import paper_1910_12308_amd as swarm
    return swarm
