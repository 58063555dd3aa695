import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library)")


@pytest.fixture(scope="session")
def windq():
    """The ctypes binding, with the in-tree HIP library loaded (fails loudly if it
    has not been built)."""
    import paper_2605_26660_amd as pkg
    pkg.load()
    return pkg
