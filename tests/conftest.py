import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    # every row selection handed to the library is range-checked first (a mistake in a test then raises instead of
    # sending a kernel out of bounds)
    from paper_2605_26646_amd import binding
    binding.CHECK_ROWS = True
