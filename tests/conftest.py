import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def tool_server():
    """The serving loop forks its tool processes from a fork server; it is started here, before any test
    touches the GPU."""
    from paper_2406_00059_amd import conveyor
    conveyor.start_tool_server()


@pytest.fixture(scope="session")
def tiny_weights():
    from workloads import TINY, make_weights, SEED_BASE
    return TINY, make_weights(TINY, SEED_BASE + 0)
