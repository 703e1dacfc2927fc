import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU runner)")


@pytest.fixture(scope="session")
def c_oracle():
    from oracle.build import build, forward_c
    build()
    return forward_c


@pytest.fixture(autouse=True)
def _release_gpu_memory(request):
    """After a GPU test its tensors (up to ~150 GB in the maximum-size cases) go back to the
    driver, so that the next test does not depend on what the caching allocator still holds."""
    yield
    if request.node.get_closest_marker("gpu") is not None:
        import gc
        import torch
        gc.collect()
        torch.cuda.empty_cache()
