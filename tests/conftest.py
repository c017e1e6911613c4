import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    import torch

    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(autouse=True)
def _guard_regions(request):
    """GPU tests allocate every buffer the library writes with a patterned guard region behind
    it (harness._buf); after the test all of them must be intact."""
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    from paper_2512_02541_amd import harness

    harness.guards_enabled = True
    harness._guards.clear()
    try:
        yield
        harness.check_all_guards()
    finally:
        harness.guards_enabled = False
        harness._guards.clear()
