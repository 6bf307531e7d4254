import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs through the C-ABI HIP library)")


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(autouse=True)
def _library_switches_back_to_default():
    """The library's test switches are process-wide: whatever a test sets (or leaves set when it
    fails half-way) is undone before the next test starts."""
    yield
    try:
        from paper_2401_06197_amd import binding
        if os.path.exists(binding.LIB_PATH):
            binding.dcnv4_set_option("reset", 0)
    except Exception:
        pass
