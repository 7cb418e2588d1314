import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def gpu_lib():
    """The HIP library through its Python binding; a missing library or GPU is a
    failure of the gpu-marked tests, never a skip into some other path."""
    import torch
    from paper_1901_01544_amd import iwp
    assert torch.cuda.is_available(), "gpu-marked tests need a GPU"
    iwp.load()
    return iwp
