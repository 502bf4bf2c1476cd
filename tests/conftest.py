import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.build()
    return _oracle


def pytest_terminal_summary(terminalreporter):
    """Lines that GPU tests want in the run's summary whatever the capture mode (which comparison
    mode a full-size test used, for one)."""
    harness = sys.modules.get("gpu_harness")
    for line in getattr(harness, "SUMMARY", []):
        terminalreporter.write_line(line)
