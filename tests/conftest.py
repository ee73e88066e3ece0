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
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture
def tuning():
    """Sets tuning overrides of the library for one test (fq_set_tuning) and removes them afterwards."""
    from paper_2410_09426_amd import binding as fq
    used = []

    def set_(name, value):
        fq.fq_set_tuning(name, int(value))
        used.append(name)
    yield set_
    for name in used:
        fq.fq_set_tuning(name, None)
