"""GPU-centric feature-row gather for AMD MI355X (gfx950).

``out[i, :] = table[idx[i], :]`` with the table in pinned, GPU-mapped host
memory (or in HBM), read directly by GPU wavefronts -- the hot path of
PyTorch-Direct (arXiv 2101.07956, Sections 3 and 4.5).  The work is done by
``libud.so`` (C ABI in ``include/ud.h``); this package is its thin binding.

The compiled library is loaded on first use of any name of the binding
(``ud_gather``, ``Table``, ...), so that ``paper_2101_07956_amd.build`` can be
imported to compile it.  If the library has not been built that first use
raises ImportError: there is no fallback path.
"""
from __future__ import annotations

import importlib

__all__ = ["binding", "table", "build"]


def __getattr__(name: str):
    if name.startswith("__"):
        raise AttributeError(name)
    if name in ("build", "tune", "binding", "table"):          # submodules: plain imports, no library needed for build
        return importlib.import_module("." + name, __name__)
    binding = importlib.import_module(".binding", __name__)
    if hasattr(binding, name):
        value = getattr(binding, name)
    else:
        table = importlib.import_module(".table", __name__)
        if not hasattr(table, name):
            raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
        value = getattr(table, name)
    globals()[name] = value          # resolved once: later look-ups do not come through here
    return value
