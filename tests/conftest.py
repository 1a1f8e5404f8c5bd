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
    """The HIP library through its Python binding; fails loudly when the
    extension is not built or no GPU is present."""
    import torch
    from paper_2206_07882_amd import qrnnt
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    qrnnt.load()
    return qrnnt
