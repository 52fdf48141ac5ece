"""CPU oracle for the feature-row gather (test infrastructure only).

Thin ctypes loader around ``gather_oracle.c``, the plain C definition of
``out[i, :] = table[idx[i], :]`` (PyTorch-Direct, Section 2.2 and Listings 1-2)
and of the request-count model of Section 4.5.  Nothing in the product path may
import this package; it exists so that tests, the smoke check and the
benchmark's ``cpu_baseline`` leg have an independent result to compare with.
It imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gather_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, F16, F16_TO_F32 = 0, 1, 2
I64, I32 = 0, 1
OK, ERR_INVALID_ARG, ERR_INDEX = 0, 1, 4


class OracleIndexError(IndexError):
    """An entry of the ID list lies outside [0, N); ``pos`` is its position."""

    def __init__(self, pos: int):
        super().__init__(f"index out of range at position {pos}")
        self.pos = pos


def build(force: bool = False) -> str:
    """Compile the oracle with the host C compiler (no HIP involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", _SRC, "-o", _LIB, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_f16_bits_to_f32_bits.restype = ctypes.c_uint32
        lib.oracle_f16_bits_to_f32_bits.argtypes = [ctypes.c_uint16]
        lib.oracle_gather.restype = ctypes.c_int
        lib.oracle_gather.argtypes = [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
            ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64),
        ]
        lib.oracle_gather_pitched.restype = ctypes.c_int
        lib.oracle_gather_pitched.argtypes = [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
            ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64),
        ]
        lib.oracle_scatter.restype = ctypes.c_int
        lib.oracle_scatter.argtypes = [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
            ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64),
        ]
        lib.oracle_scatter_pitched.restype = ctypes.c_int
        lib.oracle_scatter_pitched.argtypes = [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
            ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64),
        ]
        lib.oracle_count_requests.restype = ctypes.c_int64
        lib.oracle_count_requests.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
        ]
        lib.oracle_circular_shift.restype = ctypes.c_int64
        lib.oracle_circular_shift.argtypes = [ctypes.c_int64] * 4
        _lib = lib
    return _lib


_TABLE_NP = {F32: (np.uint32, np.uint32), F16: (np.uint16, np.uint16), F16_TO_F32: (np.uint16, np.uint32)}


def gather_raw(table_ptr: int, N: int, D: int, dtype: int, idx: np.ndarray, out: np.ndarray,
               pitch: int | None = None) -> None:
    """Oracle gather from a raw host address (for tables that live in pinned memory).

    ``pitch`` is the distance between rows in elements (default ``D``: a dense table)."""
    itype = {np.dtype(np.int64): I64, np.dtype(np.int32): I32}[idx.dtype]
    assert idx.flags.c_contiguous and out.flags.c_contiguous
    bad = ctypes.c_int64(-1)
    if pitch is None:
        rc = _load().oracle_gather(table_ptr, N, D, dtype, idx.ctypes.data, itype, idx.size,
                                   out.ctypes.data, ctypes.byref(bad))
    else:
        rc = _load().oracle_gather_pitched(table_ptr, N, D, pitch, dtype, idx.ctypes.data, itype, idx.size,
                                           out.ctypes.data, ctypes.byref(bad))
    if rc == ERR_INDEX:
        raise OracleIndexError(bad.value)
    if rc != OK:
        raise ValueError(f"oracle_gather: invalid argument (status {rc})")


def gather(table: np.ndarray, idx: np.ndarray, dtype: int | None = None) -> np.ndarray:
    """``out[i, :] = conv(table[idx[i], :])`` on bit patterns.

    ``table`` is a C-contiguous 2-D array of 4-byte (float32/uint32/int32) or
    2-byte (float16/uint16) elements; ``idx`` a 1-D int64 or int32 array.
    ``dtype`` defaults to the same-width copy; pass ``F16_TO_F32`` for the
    widening gather.  The result has the table's dtype (float32 when widening).
    """
    assert table.ndim == 2 and table.flags.c_contiguous
    idx = np.ascontiguousarray(idx)
    assert idx.ndim == 1
    if dtype is None:
        dtype = F32 if table.dtype.itemsize == 4 else F16
    in_bits, out_bits = _TABLE_NP[dtype]
    assert table.dtype.itemsize == np.dtype(in_bits).itemsize
    N, D = table.shape
    out = np.empty((idx.size, D), dtype=out_bits)
    gather_raw(table.ctypes.data, N, D, dtype, idx, out)
    if dtype == F16_TO_F32:
        return out.view(np.float32)
    return out.view(table.dtype)


def scatter_raw(table_ptr: int, N: int, D: int, dtype: int, idx: np.ndarray, src: np.ndarray,
                pitch: int | None = None) -> None:
    """Oracle scatter into a table at a raw host address: ``table[idx[i], :] = src[i, :]``, in order of i.
    ``pitch`` is the distance between table rows in elements (default ``D``)."""
    itype = {np.dtype(np.int64): I64, np.dtype(np.int32): I32}[idx.dtype]
    assert idx.flags.c_contiguous and src.flags.c_contiguous
    bad = ctypes.c_int64(-1)
    rc = _load().oracle_scatter_pitched(table_ptr, N, D, D if pitch is None else pitch, dtype, idx.ctypes.data, itype,
                                        idx.size, src.ctypes.data, ctypes.byref(bad))
    if rc == ERR_INDEX:
        raise OracleIndexError(bad.value)
    if rc != OK:
        raise ValueError(f"oracle_scatter: invalid argument (status {rc})")


def scatter(table: np.ndarray, idx: np.ndarray, src: np.ndarray) -> None:
    """In place: ``table[idx[i], :] = src[i, :]`` for i = 0, 1, ... (the last duplicate wins)."""
    assert table.ndim == 2 and table.flags.c_contiguous and table.flags.writeable
    assert src.dtype.itemsize == table.dtype.itemsize and src.shape == (idx.size, table.shape[1])
    idx = np.ascontiguousarray(idx)
    src = np.ascontiguousarray(src)
    dtype = F32 if table.dtype.itemsize == 4 else F16
    scatter_raw(table.ctypes.data, table.shape[0], table.shape[1], dtype, idx, src)


def f16_bits_to_f32_bits(h: np.ndarray) -> np.ndarray:
    """Element-wise binary16 -> binary32 widening on raw bit patterns."""
    lib = _load()
    h = np.asarray(h, dtype=np.uint16)
    flat = h.ravel()
    out = np.empty(flat.shape, dtype=np.uint32)
    for k in range(flat.size):
        out[k] = lib.oracle_f16_bits_to_f32_bits(int(flat[k]))
    return out.reshape(h.shape)


def circular_shift(i: int, r: int, D: int, elems_per_line: int) -> int:
    return _load().oracle_circular_shift(i, r, D, elems_per_line)


def count_requests(rows, shift, D: int, elem_bytes: int, W: int, line_bytes: int,
                   row_lo: int = 0, row_hi: int | None = None) -> int:
    """Distinct (warp, line) pairs touched by output rows [row_lo, row_hi) (Section 4.5)."""
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    M = rows.size
    if row_hi is None:
        row_hi = M
    sp = None
    if shift is not None:
        shift = np.ascontiguousarray(shift, dtype=np.int64)
        assert shift.size == M
        sp = shift.ctypes.data
    n = _load().oracle_count_requests(rows.ctypes.data, sp, M, D, elem_bytes, W, line_bytes, row_lo, row_hi)
    if n < 0:
        raise ValueError("oracle_count_requests: invalid argument")
    return int(n)
