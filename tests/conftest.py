import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


@pytest.fixture(scope="session")
def lib():
    """The GPU binding; GPU tests fail loudly if the HIP library is missing."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this process")
    import paper_2605_26845_amd as moe
    moe.load()
    return moe


@pytest.fixture(scope="session")
def hostlib():
    """The binding for its host-only entry points (no GPU needed: nothing is enqueued)."""
    import paper_2605_26845_amd as moe
    import os
    if not os.path.exists(moe._LIB_PATH):
        moe.build()
    moe.load()
    return moe
