import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle

    _oracle.build()
    return _oracle


@pytest.fixture(scope="session")
def dlrt():
    """The ctypes binding over the HIP library; GPU tests call the C ABI through it."""
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    from paper_2207_08820_amd import binding

    binding.load()
    return binding
