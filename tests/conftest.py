import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests print their case before running so a box lost to a fault names it.
    pass


@pytest.fixture(scope="session")
def gpu_lib():
    """The loaded C-ABI binding; fails loudly if the HIP library is not built."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    import paper_2405_18832_amd as moe
    moe.load()      # raises if the extension is missing
    return moe
