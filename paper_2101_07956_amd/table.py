"""Small conveniences over the C-ABI binding for callers that hold torch tensors.

Marshalling only: pointer extraction, shape bookkeeping, output allocation.
"""
from __future__ import annotations

import ctypes

import numpy as np

from . import binding as B

_ELEM_NP = {B.UD_F32: np.float32, B.UD_F16: np.float16}


class Table:
    """A feature table owned by the library (pinned host memory, or HBM after ``to_device``)."""

    def __init__(self, N: int, D: int, elem: int = B.UD_F32, flags: int = B.UD_TABLE_COHERENT, _handle=None):
        self.handle = _handle if _handle is not None else B.ud_alloc_table(N, D, elem, flags)
        self.N, self.D, self.elem = B.ud_table_shape(self.handle)
        self.pitch = B.ud_table_pitch(self.handle)          # elements between rows (> D for padded tables)
        self.device_ptr = B.ud_table_device_ptr(self.handle)
        self.host_ptr = B.ud_table_host_ptr(self.handle)

    @property
    def elem_bytes(self) -> int:
        return 4 if self.elem == B.UD_F32 else 2

    @property
    def nbytes(self) -> int:
        return self.N * self.pitch * self.elem_bytes

    def numpy(self) -> np.ndarray:
        """The CPU's view of a host table (no copy): the CPU uses it like ordinary memory.
        For a padded table this is the [N, D] data window of the [N, pitch] storage."""
        if not self.host_ptr:
            raise ValueError("device-resident table has no host view")
        buf = (ctypes.c_char * self.nbytes).from_address(self.host_ptr)
        return np.frombuffer(buf, dtype=_ELEM_NP[self.elem]).reshape(self.N, self.pitch)[:, : self.D]

    def to_device(self, row0: int = 0, n: int | None = None) -> "Table":
        n = self.N - row0 if n is None else n
        return Table(0, 0, _handle=B.ud_table_to_device(self.handle, row0, n))

    def free(self) -> None:
        if self.handle:
            B.ud_free_table(self.handle)
            self.handle = None

    def __del__(self):  # pragma: no cover - best effort
        try:
            self.free()
        except Exception:
            pass


class Cache:
    """HBM copies of chosen rows of a host table plus the row -> slot map (hybrid placement)."""

    def __init__(self, table: Table, hot_rows: np.ndarray):
        hot_rows = np.ascontiguousarray(hot_rows, dtype=np.int64)
        self.table = table                      # keeps the host table alive
        self.n_hot = int(hot_rows.size)
        self.handle = B.ud_cache_create(table.handle, hot_rows.ctypes.data, hot_rows.size)

    def free(self) -> None:
        if self.handle:
            B.ud_cache_free(self.handle)
            self.handle = None

    def __del__(self):  # pragma: no cover - best effort
        try:
            self.free()
        except Exception:
            pass


def gather(table: Table, idx, out=None, widen: bool = False, tuning: B.ud_tuning | None = None, check: bool = False):
    """``out[i, :] = table[idx[i], :]`` for a torch int64/int32 tensor ``idx`` in GPU memory, or in pinned host
    memory (the kernel then reads the IDs over the link like the rows: no copy, worth it for small batches).

    Enqueues on torch's current stream and returns the output tensor (allocated
    here when ``out`` is None).  ``widen`` turns an fp16 table into fp32 output.
    ``check`` waits and raises ``UdIndexError`` on an out-of-range ID.
    """
    import torch

    assert (idx.is_cuda or idx.is_pinned()) and idx.dim() == 1 and idx.is_contiguous()
    device = idx.device if idx.is_cuda else torch.device("cuda", torch.cuda.current_device())
    itype = {torch.int64: B.UD_I64, torch.int32: B.UD_I32}[idx.dtype]
    if table.elem == B.UD_F32:
        dtype, odt = B.UD_F32, torch.float32
    elif widen:
        dtype, odt = B.UD_F16_TO_F32, torch.float32
    else:
        dtype, odt = B.UD_F16, torch.float16
    M = idx.numel()
    if out is None:
        out = torch.empty((M, table.D), dtype=odt, device=device)
    assert out.is_cuda and out.is_contiguous() and out.dtype == odt and out.numel() == M * table.D
    stream = torch.cuda.current_stream(device).cuda_stream
    if table.pitch != table.D:
        assert tuning is None, "explicit tuning is for dense tables"
        B.ud_gather_pitched(table.device_ptr, table.N, table.D, table.pitch, dtype, idx.data_ptr(), itype, M,
                            out.data_ptr(), stream)
    else:
        B.ud_gather_tuned(table.device_ptr, table.N, table.D, dtype, idx.data_ptr(), itype, M,
                          out.data_ptr(), stream, tuning)
    if check:
        B.ud_gather_status(stream)
    return out
