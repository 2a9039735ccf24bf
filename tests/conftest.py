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
    """The loaded C-ABI binding; fails loudly if the HIP library is not built."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2512_07710_amd as moe
    moe.load_library()
    return moe
