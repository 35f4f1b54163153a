import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """Keep the no-allocation entry point's test last: it shares a per-device scratch
    array with nothing else, but a failure there must not hide the other GPU tests."""
    items.sort(key=lambda it: ("test_zz_" in it.nodeid, 0))
