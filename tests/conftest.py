import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "production_rings: run with the library's own ring length instead of the tests' short rings")


@pytest.fixture(autouse=True)
def _short_rings(request, monkeypatch):
    """The streams between operations are rings of at least 8,192 elements in production; the test traces are mostly
    shorter than that, so the tests run with the smallest rings the plan allows (1,024 elements, or what the widest
    batch group needs) and wrap them many times.  Tests marked `production_rings` (the full-length workloads) keep
    the library's own choice."""
    if request.node.get_closest_marker("production_rings") is None:
        monkeypatch.setenv("EST_RING_ELEMS", "1024")
