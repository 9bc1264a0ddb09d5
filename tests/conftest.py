import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


NEEDS_LIBRARY = ("test_abi", "test_ordering_native", "test_gpu_", "test_zz_no_alloc")


@pytest.fixture(scope="session")
def _library():
    """Builds the in-tree shared library if it is not there yet."""
    from paper_2101_08358_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2101_08358_amd import build
        build.build()
    return binding.library_path()


@pytest.fixture(autouse=True)
def _built_library(request):
    """Only the tests that load the library ask for it: the oracle's pins run where hipcc is absent."""
    name = os.path.basename(str(request.node.fspath))
    if name.startswith(NEEDS_LIBRARY):
        request.getfixturevalue("_library")
    yield
