import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _have_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture
def lane_per_row():
    """For tests about the row-per-lane kernels (segment codes built in registers, slot order, bf16
    storage, bit-identity of their variants): small batches of short rows, which the library
    would give sixteen threads per row (`thread_per_sample_1d_rows`), are kept on those kernels."""
    import paper_2204_03643_amd as tv
    saved = tv.tv_dispatch_threshold("thread_per_sample_1d_rows")
    tv.tv_dispatch_override("thread_per_sample_1d_rows", 0)
    yield
    tv.tv_dispatch_override("thread_per_sample_1d_rows", saved)
