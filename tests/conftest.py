import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X")
    config.addinivalue_line("markers", "tuned_only: runs once, on the tuned kernels (not on both kernel paths)")


def _have_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture
def decode_chunks():
    """Setter of the library's thread-local test switch "at least n chunks per row of the tuned
    decode" (cq_bench.h); automatic again after the test."""
    from paper_2502_14882_amd import binding as cq
    yield cq.cq_bench_set_decode_chunks
    cq.cq_bench_set_decode_chunks(0)
