import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def svip():
    """The HIP path through its Python binding; fails loudly if the library is missing."""
    import torch

    assert torch.cuda.is_available(), "gpu-marked test run without a GPU"
    import paper_2411_18462_amd as pkg

    pkg.load()  # raises if libsvip.so is not built
    return pkg
