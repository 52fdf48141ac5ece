import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    _build_if_nothing_is_built()


def _build_if_nothing_is_built():
    """The tests load the in-tree libraries as built; only a tree with no library at all is built first
    (hipcc cross-compiles without a GPU).  After changing a source, rebuild before running the tests."""
    pkg = os.path.join(ROOT, "paper_2101_07956_amd")
    if all(os.path.exists(os.path.join(pkg, lib)) for lib in ("libud.so", "libud_baseline.so")):
        return
    from paper_2101_07956_amd import build as hip_build
    hip_build.build(verbose=False)


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped, not failed, where no GPU is visible."""
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
