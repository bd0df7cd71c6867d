import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture
def progress(capsys):
    """print() that pytest does not capture, so that a long test shows its steps while it runs."""
    def say(msg):
        with capsys.disabled():
            print(f"\n[progress] {msg}", end="", flush=True)
    return say
