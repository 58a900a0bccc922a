import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def orc():
    from oracle import oracle

    oracle.build()
    return oracle


@pytest.fixture(scope="session")
def built_library():
    """libcapmoe.so: what is built is loaded; it is compiled only if nothing is there."""
    from paper_2503_05066_amd import build, capmoe

    if not os.path.exists(capmoe.LIB_PATH):
        build.build()
    return capmoe.load()
