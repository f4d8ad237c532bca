import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture
def progress(capsys):
    """print() that reaches the terminal although output is captured: tests that run for minutes
    report every step, so that a harness watching for silence does not take them for hung"""
    def emit(*args, **kwargs):
        with capsys.disabled():
            print(*args, **kwargs, flush=True)
    return emit


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
