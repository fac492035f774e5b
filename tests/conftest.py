import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped, loudly, when no GPU is visible (e.g. `pytest tests/` on a CPU machine)."""
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture
def launch_override():
    """force(name, value): force one launch-shape choice of the library (pz_debug_set_launch_override) for the
    rest of the test; every override is handed back to the library afterwards."""
    import paper_2602_11937_amd as pz
    used = []

    def force(name, value):
        used.append(name)
        pz.pz_debug_set_launch_override(name, value)

    yield force
    for name in used:
        pz.pz_debug_set_launch_override(name, -1)
