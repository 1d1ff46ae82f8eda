import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture
def mecefo_option():
    """Sets library switches (mecefo_set_option) for one test and puts them back to "auto" afterwards."""
    from paper_2510_16415_amd import binding as B
    changed = []

    def set_option(name, value):
        B.mecefo_set_option(name, value)
        changed.append(name)

    yield set_option
    for name in changed:
        B.mecefo_set_option(name, "auto")
