import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C ABI of libmcsd.so)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped automatically where no GPU is visible, so that a plain
    # `pytest tests/` on a CPU-only machine stays green.
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture
def plan_override():
    """Forces the launch plan of the matrix-core attention kernel for one test (kernel variant,
    segment length, item target) through mcsd_attn_plan_override; automatic again afterwards."""
    from paper_2401_06706_amd import binding as M
    yield M.mcsd_attn_plan_override
    M.mcsd_attn_plan_override(0, 0, 0)
