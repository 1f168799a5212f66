import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(autouse=True)
def _separate_kernels_by_default():
    """The test workloads are small, and on small calls the fused entry point runs everything in one launch
    (HG_OPT_FUSED_KERNEL = 0).  The tests of the separate kernels, their options and their partitions therefore pin
    new contexts to the separate kernels; tests of the single launch, and the full-size tests, which run the library's
    defaults, set the option themselves."""
    from paper_2402_05099_amd import binding as hb
    old = dict(hb.Context.default_options)
    hb.Context.default_options = {hb.HG_OPT_FUSED_KERNEL: 1}
    yield
    hb.Context.default_options = old
