import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    # the tests load the libraries that are built; only when there are none they are compiled first
    from paper_2212_05339_amd.build import ensure_built
    ensure_built()


def _have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    # GPU tests are selected with -m gpu; if they are collected on a machine without a GPU
    # (plain `pytest tests/`), skip them instead of failing.
    if any("gpu" in it.keywords for it in items) and not _have_gpu():
        skip = pytest.mark.skip(reason="no GPU on this machine")
        for it in items:
            if "gpu" in it.keywords:
                it.add_marker(skip)
