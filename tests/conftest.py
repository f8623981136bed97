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


@pytest.fixture
def eq_override():
    """Sets kernel-selection overrides of the library (csrc/eq_testing.h) and clears them all afterwards."""
    import paper_2403_02775_amd as eqg
    yield eqg.set_override
    for which in range(5):
        eqg.set_override(which, 0)
