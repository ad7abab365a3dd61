import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    oracle.build()
    return oracle


@pytest.fixture(autouse=True)
def _default_decode_plan():
    """Tests that change the decode plan of their calls do not leak it into the next test."""
    yield
    import sys
    gpu_utils = sys.modules.get("gpu_utils")
    if gpu_utils is not None:
        gpu_utils.planned.reset()
