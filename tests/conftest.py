import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, where no GPU is visible.
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture
def options():
    """Setter for the library's process-wide test hooks (lococo_debug_option); all of them are back
    at their defaults when the test ends."""
    from paper_2406_05317_amd import binding as lb
    lb.lococo_debug_option(lb.LOCOCO_OPT_RESET)
    yield lb.lococo_debug_option
    lb.lococo_debug_option(lb.LOCOCO_OPT_RESET)
