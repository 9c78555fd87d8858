import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture
def tuning():
    """set(knob, value) overrides one choice of the library's host-side plan (sdkde_set_tuning, a test hook of the
    C ABI) for the duration of the test; every knob is restored afterwards."""
    import paper_2602_10378_amd as P
    touched = []

    def set_knob(knob, value):
        touched.append(knob)
        P.sdkde_set_tuning(knob, value)

    yield set_knob
    for knob in touched:
        P.sdkde_set_tuning(knob, 0)
