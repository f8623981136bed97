import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# The pins themselves are tested by running them against copies of the oracle with a planted
# mistake (test_pins_catch_mistakes.py): that directory's `oracle` package then comes first.
_ALT = os.environ.get("EASYQUANT_ORACLE_UNDER_TEST")
if _ALT:
    sys.path.insert(0, _ALT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "oracle_pool: recomputes many rows with the oracle in worker processes")


# The oracle's worker processes (oracle/rowpool.py) are started right after collection, i.e. before
# any test has run and therefore before the first GPU call of this process.
_POOL = None


def _make_pool():
    global _POOL
    if _POOL is None:
        from oracle.rowpool import RowPool
        _POOL = RowPool(min(14, os.cpu_count() or 1))
    return _POOL


def pytest_collection_finish(session):
    if session.config.option.collectonly:
        return
    if any(item.get_closest_marker("oracle_pool") for item in session.items):
        _make_pool()


def pytest_sessionfinish(session, exitstatus):
    global _POOL
    if _POOL is not None:
        _POOL.close()
        _POOL = None


@pytest.fixture(scope="session")
def oracle_pool():
    return _make_pool()


@pytest.fixture
def eq_override():
    """Sets kernel-selection overrides of the library (csrc/eq_testing.h) and clears them all afterwards."""
    import paper_2403_02775_amd as eqg
    yield eqg.set_override
    for which in range(eqg.OVR_COUNT):
        eqg.set_override(which, 0)
