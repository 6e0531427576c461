import os
import sys

import pytest
from hypothesis import settings

# property tests draw the same examples on every run
settings.register_profile("repeatable", derandomize=True, deadline=None)
settings.load_profile("repeatable")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI on cuda:0)")
