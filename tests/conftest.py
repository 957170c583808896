import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _library_is_built():
    """Tests load the library that is built in-tree and compile it only when there is none."""
    from paper_1906_11024_amd import binding as sb
    if not os.path.exists(sb.LIB_PATH):
        from paper_1906_11024_amd import build
        build.build(verbose=False)
