import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _recompute_count(n_ctx, num, den):
    """p = r * n of Eq. 3 for the shared workload generator: the oracle's count, checked against the library's own
    host routine (the library loads without a GPU); a disagreement is an error right here."""
    from oracle import a3_oracle as ora
    k = ora.recompute_count(n_ctx, num, den)
    try:
        from paper_2511_17560_amd import api
        k_lib = api.a3_recompute_count(n_ctx, num, den)
    except RuntimeError:          # library not built: oracle-only test runs
        k_lib = k
    assert k == k_lib, (n_ctx, num, den, k, k_lib)
    return k


import a3_synth  # noqa: E402

a3_synth.use_recompute_count(_recompute_count)


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
