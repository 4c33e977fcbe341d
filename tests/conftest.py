import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_lib():
    from oracle import oracle
    return oracle.default()


# The full-size GPU tests compare sampled rows with the CPU oracle, which runs in worker processes.
# They are forked here, when collection has finished and before any test touches the GPU.
_POOL = None


def pytest_collection_finish(session):
    global _POOL
    if _POOL is None and any(item.get_closest_marker("gpu") for item in session.items):
        from oracle.pool import OraclePool
        _POOL = OraclePool(max(1, min(16, os.cpu_count() or 1)))


def pytest_sessionfinish(session, exitstatus):
    global _POOL
    if _POOL is not None:
        _POOL.close()
        _POOL = None


@pytest.fixture(scope="session")
def oracle_pool():
    assert _POOL is not None, "the oracle's worker pool is created when GPU tests are collected"
    return _POOL
