import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _oracle_built():
    """The checker is plain C; build it if the shared object is not there yet."""
    so = os.path.join(ROOT, "oracle", "libabft_oracle.so")
    if not os.path.exists(so):
        sys.path.insert(0, os.path.join(ROOT, "oracle"))
        from oracle import build as _b
        _b.build()
    yield
