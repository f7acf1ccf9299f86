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


@pytest.fixture(params=[1, 2, 3], ids=["spread", "neighbours", "timed"])
def tile_order(request, monkeypatch):
    """Runs a test once per order in which the encode kernel's workgroups take tiles (the buckets
    must be the same bytes either way): every plan the test makes gets the order set."""
    from paper_2605_06534_amd import binding
    make = binding.shard_plan

    def planned(*a, **kw):
        plan = make(*a, **kw)
        plan.set_tile_order(request.param)
        return plan

    monkeypatch.setattr(binding, "shard_plan", planned)
    return request.param
