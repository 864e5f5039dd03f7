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
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(autouse=True)
def _guard_bands_stay_intact(request):
    """After every GPU test: the 4 KB guard bands around the buffers the test handed to the library (cache, decode
    workspace, score buffer, chunk workspace; allocated through PodCache(..., guard_bytes=4096)) still hold their
    pattern, i.e. no kernel wrote outside what it was given."""
    yield
    if "gpu" in request.keywords and _have_gpu():
        import paper_2412_02252_amd as pod
        bad = pod.guards_intact()
        assert not bad, f"guard bands overwritten: {bad}"
