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
    """The tests load the in-tree libraries as built.  A tree with no library, or with libraries whose build
    stamp does not match the sources as they are now (an edit since the last build), is built first: hipcc
    cross-compiles without a GPU, and a parity run must belong to the code in the tree."""
    from paper_2101_07956_amd import build as hip_build
    hip_build.ensure_built(verbose=False)


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


class RawStreams:
    """n distinct HIP streams (default priority) made with hipStreamCreate: torch hands out streams from a
    pool of 32 per device, so torch.cuda.Stream() objects cannot exceed the library's 63 per-stream slots."""

    def __init__(self, n):
        import ctypes
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipStreamCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipStreamDestroy.argtypes = [ctypes.c_void_p]
        self.handles = []
        for _ in range(n):
            h = ctypes.c_void_p()
            assert self.hip.hipStreamCreate(ctypes.byref(h)) == 0
            self.handles.append(h.value)
        assert len(set(self.handles)) == n

    def close(self):
        for h in self.handles:
            assert self.hip.hipStreamDestroy(h) == 0
        self.handles = []
