import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def npas():
    """The Python binding of the HIP library (built beforehand, in-tree)."""
    import paper_2012_00596_amd as pkg
    return pkg


@pytest.fixture
def force_variant(npas):
    """Overrides the library's kernel / format choice for one test (the NPAS_FORCE_VARIANT switch)."""
    yield lambda name: npas.set_switches(name)
    npas.set_switches(None)
