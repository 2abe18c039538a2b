import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _built_libraries():
    """Use the libraries that are built; compile only when one is missing."""
    import __graft_entry__ as entry
    if not os.path.exists(entry.LIB):
        entry.build_library()
    import oracle
    oracle.build()
