import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def lib():
    """The ctypes binding over the C-ABI library (built in-tree if absent)."""
    from paper_2410_18311_amd import build as _build
    if not os.path.exists(_build.LIB_PATH):
        _build.build_library()
    from paper_2410_18311_amd import coreinfer
    return coreinfer


def gpu_available() -> bool:
    import torch
    return torch.cuda.is_available()
