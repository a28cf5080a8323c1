import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def paro():
    """The product binding.  The library is built first if it has never been built; if that
    fails the import below raises - there is no fallback to run the tests against."""
    from __graft_entry__ import ensure_built
    ensure_built()
    import paper_2310_06003_amd as paro_mod
    return paro_mod
