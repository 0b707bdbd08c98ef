import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def mbq():
    """The Python binding over the HIP library; GPU tests only."""
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    import paper_2602_20191_amd as pkg

    pkg.load()  # raises if the HIP library is missing: no silent fallback
    return pkg
