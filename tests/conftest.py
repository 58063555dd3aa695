import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

_POOL = None


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library)")
    config.addinivalue_line("markers", "oracle_pool: checks many units against the oracle, in worker processes")


def pytest_collection_finish(session):
    """Worker processes for the oracle (it is single-threaded numpy; the stack tests check a hundred units).
    They are started here, before any test has touched the GPU: a process that has initialised the GPU must not
    start other programs.  The workers import numpy and the oracle only."""
    global _POOL
    if _POOL is None and any(item.get_closest_marker("oracle_pool") for item in session.items):
        import multiprocessing as mp
        n = max(1, min(16, os.cpu_count() or 1))
        try:
            _POOL = mp.get_context("spawn").Pool(n)
            _POOL.map(abs, range(n))
        except Exception:           # the tests then run the oracle in this process, on smaller samples
            _POOL = None


def pytest_unconfigure(config):
    global _POOL
    if _POOL is not None:
        _POOL.close()
        _POOL = None


@pytest.fixture(scope="session")
def oracle_pool():
    return _POOL


@pytest.fixture(scope="session")
def windq():
    """The ctypes binding, with the in-tree HIP library loaded (fails loudly if it
    has not been built)."""
    import paper_2605_26660_amd as pkg
    pkg.load()
    return pkg
