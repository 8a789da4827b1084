import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture
def debug_knobs():
    """Sets debug settings of the library (ap_debug_set) for one test and restores the defaults afterwards."""
    from paper_2511_00855_amd import binding as B
    yield B.debug_set
    B.debug_reset()
