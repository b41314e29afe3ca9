import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def cam():
    """The HIP library behind its Python binding; GPU tests fail loudly when it is missing."""
    import torch
    from paper_2508_02322_amd import binding
    assert torch.cuda.is_available(), "GPU test selected but no GPU is visible"
    return binding.Camera(device=0)
