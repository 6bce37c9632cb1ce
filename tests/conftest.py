import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _oracle_built():
    import oracle
    oracle.build()


@pytest.fixture(scope="session", autouse=True)
def _library_built():
    """The tests load the library that is built; only when there is none do they build it
    (the product itself never builds or falls back: binding.lib() raises)."""
    from paper_2509_19729_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
