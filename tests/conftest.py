import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: a GPU case that follows a workload for thousands of steps (minutes, "
                                       "mostly the CPU oracle's); still part of -m gpu")


@pytest.fixture(scope="session")
def mkv():
    """The Python binding over the C-ABI library; GPU tests only."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    import paper_2605_29873_amd.binding as b
    b.load()          # raises if the HIP library has not been built: never falls back
    return b
