import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
for _p in (ROOT, os.path.join(ROOT, "tests")):
    if _p not in sys.path:
        sys.path.insert(0, _p)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP path through the C-ABI)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are selected with -m gpu; when they are selected on a machine without a GPU
    # they fail loudly in the binding rather than being skipped here.
    pass
