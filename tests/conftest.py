import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import oracle as O
    O.lib()
    return O


@pytest.fixture(scope="session")
def P(request):
    """The package with its C-ABI library loaded.  GPU tests (marker `gpu`) also require the device:
    there is no fallback to run them on."""
    import paper_2601_09212_amd as pkg
    pkg.binding.lib()
    return pkg


@pytest.fixture(autouse=True)
def _gpu_tests_need_the_gpu(request):
    if request.node.get_closest_marker("gpu") is not None:
        import torch
        assert torch.cuda.is_available(), "these tests need the MI355X"
