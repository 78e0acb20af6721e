import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X; run with -m gpu")


@pytest.fixture(scope="session")
def lib():
    """The HIP library binding; fails loudly if the shared object is not built."""
    import paper_2411_16102_amd as pkg
    return pkg.load()
