import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
HERE = os.path.dirname(os.path.abspath(__file__))
if HERE not in sys.path:
    sys.path.insert(0, HERE)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def gpu_lib():
    """The C-ABI library, loaded through the Python binding.  Fails loudly when it is not built."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this process")
    from paper_2510_08055_amd import binding
    binding.load()
    return binding
