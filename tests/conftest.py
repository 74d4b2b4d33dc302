import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


import pytest


@pytest.fixture(autouse=True)
def _release_cached_memory(request):
    """After every GPU test: give torch's cached pinned-host and device blocks back, so that the
    tests with large pinned weight tables do not run into the box's pinned-memory limit."""
    yield
    if request.node.get_closest_marker("gpu") is None:
        return
    import gc

    import torch
    gc.collect()
    if torch.cuda.is_available():
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        if hasattr(torch._C, "_host_emptyCache"):
            torch._C._host_emptyCache()
