import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
HERE = os.path.dirname(os.path.abspath(__file__))
if HERE not in sys.path:
    sys.path.insert(0, HERE)


def pytest_configure(config):
    import __graft_entry__
    __graft_entry__.ensure_built()          # compiles only when no library has been built yet
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # A GPU test on a box without a GPU is an error of the run, not a skip: it is
    # deselected by `-m "not gpu"` on CPU machines, and must really run under `-m gpu`.
    pass


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(HERE, "golden")
