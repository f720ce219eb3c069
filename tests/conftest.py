import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP path through the C-ABI)")


@pytest.fixture(scope="session")
def repo_root():
    return ROOT


@pytest.fixture
def say(capsys):
    """Progress lines of long tests, written past pytest's capture so that a run that is watched from outside (a GPU
    box kills a command that prints nothing for minutes) sees them while the test is still running."""
    def _say(*a):
        with capsys.disabled():
            print(*a, flush=True)
    return _say
