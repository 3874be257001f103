import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _libraries_built():
    """The tests load what is built; only a tree with nothing built is compiled first."""
    from paper_2410_14803_amd import build as hip_build
    hip_build.ensure_built()


@pytest.fixture(scope="session")
def oracle():
    import oracle as _o
    _o._load()
    return _o
