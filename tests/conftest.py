import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture
def tuning():
    """tuning(field=value, ...): layout choices (gss_tuning) for every GPU sampler the parity helpers create in this test."""
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import parity_util
    yield parity_util.set_tuning
    parity_util.set_tuning()
