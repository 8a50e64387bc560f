import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
for _p in (ROOT, os.path.join(ROOT, "tests")):
    if _p not in sys.path:
        sys.path.insert(0, _p)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP path through the C ABI)")


@pytest.fixture
def say(capsys):
    """Print a progress line that pytest's capture does not swallow."""
    def _say(*a):
        with capsys.disabled():
            print(*a, flush=True)
    return _say
