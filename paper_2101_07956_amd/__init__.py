"""GPU-centric feature-row gather for AMD MI355X (gfx950).

``out[i, :] = table[idx[i], :]`` with the table in pinned, GPU-mapped host
memory (or in HBM), read directly by GPU wavefronts -- the hot path of
PyTorch-Direct (arXiv 2101.07956, Sections 3 and 4.5).  The work is done by
``libud.so`` (C ABI in ``include/ud.h``); this package is its thin binding.
Importing it fails loudly if the library has not been built.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, UdError, UdIndexError, ud_tuning  # noqa: F401
from .table import Table, gather  # noqa: F401
