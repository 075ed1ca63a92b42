import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


@pytest.fixture(scope="session")
def c0():
    from synth import get_config
    return get_config("c0_tiny_f32")


def pytest_collection_modifyitems(config, items):
    try:
        import torch
        ok = torch.cuda.is_available()
    except Exception:
        ok = False
    if ok:
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
