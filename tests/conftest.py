import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu through the GPU runner)")


def pytest_terminal_summary(terminalreporter):
    from tests import helpers
    for key in sorted(helpers.SEEN, key=str):
        terminalreporter.write_line(f"[largest seen] {key}: {helpers.SEEN[key]:.3e}")


@pytest.fixture(scope="session")
def oracle():
    import oracle as o
    o.build()
    return o
