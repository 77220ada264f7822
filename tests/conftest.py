import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tslt():
    """The Python binding over the C-ABI library; fails loudly when the library is not built."""
    from paper_2512_16273_amd import tslt as mod
    mod.load()
    return mod
