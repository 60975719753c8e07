import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "big: the 2-billion-token datastore (set REST_BIG=1)")


def pytest_collection_modifyitems(config, items):
    if os.environ.get("REST_BIG") == "1":
        return
    skip_big = pytest.mark.skip(reason="full-size workload; set REST_BIG=1 to run")
    for item in items:
        if "big" in item.keywords:
            item.add_marker(skip_big)
