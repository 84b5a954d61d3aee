import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def ensure_built():
    """Load what is built; build only if nothing is."""
    from paper_2602_06079_amd import build as _build
    if not os.path.exists(_build.OUT) or not os.path.exists(_build.EXAMPLE_OUT):
        _build.build()
    return _build.OUT


@pytest.fixture(scope="session")
def canz():
    ensure_built()
    from paper_2602_06079_amd import binding
    return binding
