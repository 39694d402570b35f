import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_collection_modifyitems(config, items):
    """GPU tests fail loudly (not skip) when selected on a box without a GPU; they are
    deselected by -m "not gpu" on CPU-only hosts."""
    return


@pytest.fixture
def score_path():
    """Pins the scoring kernels for the duration of a test (obc_set_score_path) and restores the routing by shape."""
    from paper_2510_07651_amd import binding as obc

    yield obc.obc_set_score_path
    obc.obc_set_score_path("auto")
    obc.obc_set_score_tuning(0, 0)
    obc.obc_set_sweep2_form(0)
