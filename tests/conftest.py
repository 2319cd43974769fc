import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs through the C-ABI HIP library)")


@pytest.fixture
def progress(capsys):
    """A print that reaches the terminal while the test is still running (output capture is lifted for the line):
    the long full-depth tests report their steps as they go."""
    def say(*args):
        with capsys.disabled():
            print(*args, flush=True)
    return say
