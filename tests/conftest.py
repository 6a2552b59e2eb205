import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped, not failed, on a machine without a GPU."""
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture
def plan():
    """plan(name, value) forces one of the library's kernel-plan overrides through
    qspec_debug_set_plan; every override set this way is released after the test."""
    from paper_2410_11305_amd import binding as B
    used = []

    def force(name, value):
        B.debug_set_plan(name, value)
        used.append(name)

    yield force
    for name in used:
        B.debug_set_plan(name, None)
