import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


# With one column set per head the library picks between two attention kernels by job size, and small
# test shapes would all land in one of them: these modules run every test through both.
BOTH_ATTN_KERNELS = {"test_gpu_parity", "test_gpu_random_shapes", "test_gpu_logit_range", "test_gpu_gqa",
                     "test_gpu_varlen"}


@pytest.fixture(autouse=True)
def attn_kernel(request):
    block = getattr(request, "param", 0)
    from paper_2605_20813_amd import pulsecol as pc
    old = pc.DEFAULT_ATTN_BLOCK
    pc.DEFAULT_ATTN_BLOCK = block
    yield block
    pc.DEFAULT_ATTN_BLOCK = old


def pytest_generate_tests(metafunc):
    if metafunc.module.__name__.split(".")[-1] in BOTH_ATTN_KERNELS:
        metafunc.parametrize("attn_kernel", [256, 128], indirect=True, ids=["scheduled", "plain"])
