import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def S_lib():
    """The Python binding of the HIP library, for GPU tests (fails loudly without a GPU)."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2403_00176_amd as S
    return S
