import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture
def pex_option():
    """Set planner options of libpex for one test; the values in force before are put back afterwards."""
    import paper_2510_00236_amd as pex
    saved = {}

    def set_option(name, value):
        saved.setdefault(name, pex.pex_get_option(name))
        pex.pex_set_option(name, value)

    yield set_option
    for name, value in saved.items():
        pex.pex_set_option(name, value)
