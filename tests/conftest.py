import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library through its C ABI)")


def pytest_collection_modifyitems(config, items):
    # GPU tests must fail loudly, not skip, when selected with -m gpu; without a
    # GPU in the container they are simply deselected by -m "not gpu".
    pass
