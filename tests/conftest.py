import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box)")


def gpu_available():
    return os.path.exists("/dev/kfd")


@pytest.fixture(scope="session")
def lib():
    """The C-ABI library binding; GPU tests fail loudly when the HIP library is not built."""
    import paper_2604_07609_amd as blink
    return blink
