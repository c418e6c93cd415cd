import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# what the HIP runtime will read when it starts (it reads the variable once; a later change of os.environ is not seen)
HW_QUEUES_AT_START = int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def repo_root():
    return ROOT


@pytest.fixture(scope="session")
def hw_queues_at_start():
    return HW_QUEUES_AT_START
