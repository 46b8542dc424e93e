import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _have_gpu() -> bool:
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


@pytest.fixture(params=["one_kernel", "three_pass"])
def select_form(request):
    """Runs a GPU test once with each form of the select calls: the one-kernel form
    (chained scan inside the streaming kernel) and the three-pass form (per-tile
    slots), which the library otherwise chooses by the vector's length."""
    import paper_2201_07598_amd as okt
    okt.okt_debug_slot_min_n(1 if request.param == "three_pass" else 1 << 40)
    yield request.param
    okt.okt_debug_slot_min_n(0)
