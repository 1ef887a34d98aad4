"""pytest configuration: the ``gpu`` marker and the repository root on sys.path."""
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """Skip GPU tests cleanly when no GPU is visible (they are deselected with -m "not gpu" anyway)."""
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


@pytest.fixture(scope="session", autouse=True)
def _built_libraries():
    """Use the libraries that are built; build them only if nothing is there."""
    from paper_1705_07175_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        from paper_1705_07175_amd import build as hip_build

        hip_build.build()
    import oracle

    oracle.build()
    yield
