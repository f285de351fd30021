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
def options():
    """Set process-wide library options for one test (rwkvq_set_option); restored afterwards."""
    from paper_2505_03803_amd import binding as B
    before = {}

    def set_(option, value):
        before.setdefault(option, B.rwkvq_get_option(option))
        B.rwkvq_set_option(option, value)

    yield set_
    for option, value in before.items():
        B.rwkvq_set_option(option, value)
