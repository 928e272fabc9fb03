import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture
def tuning():
    """Sets tuning values of the library for one test and restores the defaults afterwards."""
    from paper_2511_17560_amd import api
    touched = []

    def set_value(name, value):
        api.a3_set_tuning(name, int(value))
        touched.append(name)

    yield set_value
    for name in touched:
        api.a3_set_tuning(name, -1)


def _has_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
