import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def fd():
    """The ctypes binding; GPU tests fail loudly if the HIP library is not built."""
    from paper_2605_20022_amd import flexdraft
    flexdraft.load()
    return flexdraft
