import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _gpu_present():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_present():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


# values of mts_attn_tuning.kernel (include/mtserve.h)
KERNEL_STREAMING, KERNEL_PREFILL, KERNEL_PLAIN = 1, 2, 3


@pytest.fixture
def attn_tuning():
    """Sets the library's attention tuning override for one test (forced schedules and kernels)
    and resets it afterwards."""
    import paper_2604_22881_amd as mts

    def set_(**fields):
        mts.mts_attn_set_tuning(**fields)
    yield set_
    mts.mts_attn_set_tuning()
