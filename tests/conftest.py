import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def c1_workload():
    from smoe_inputs import SHAPES, make_workload
    return make_workload(SHAPES["c1"])


@pytest.fixture(autouse=True)
def _release_gpu_and_pinned_memory(request):
    """GPU tests allocate multi-GB slabs and staging buffers: give the caches back
    after each one so that a long session does not run into the box's limits."""
    yield
    if request.node.get_closest_marker("gpu") is None:
        return
    import gc
    import torch
    gc.collect()
    if torch.cuda.is_available():
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        empty_host = getattr(torch._C, "_host_emptyCache", None)
        if empty_host is not None:
            empty_host()
