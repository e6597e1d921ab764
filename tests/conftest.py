import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def built_library():
    # load what is built; compile only when nothing is (after a source change, build before running tests)
    from paper_2603_25872_amd import build
    return build.ensure_built()


@pytest.fixture(scope="session")
def orc():
    from oracle.ref import Oracle
    return Oracle(64)


@pytest.fixture(scope="session")
def orc32():
    from oracle.ref import Oracle
    return Oracle(32)
