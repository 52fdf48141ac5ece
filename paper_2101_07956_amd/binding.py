"""ctypes binding of ``libud.so`` (the C ABI declared in ``include/ud.h``).

Argument marshalling only: every step of the gather runs in the library's HIP
kernels.  The functions carry the C names; each returns the library's status
code converted to an exception (``UdError``) unless it is ``UD_OK``.  PyTorch
appears only as a source of device pointers and streams in the callers; this
module does not import it.

The library must have been built (``python -m paper_2101_07956_amd.build``);
importing fails loudly otherwise -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libud.so")

UD_OK, UD_ERR_INVALID_ARG, UD_ERR_UNSUPPORTED, UD_ERR_OOM, UD_ERR_INDEX_OUT_OF_RANGE, UD_ERR_HIP = range(6)
UD_F32, UD_F16, UD_F16_TO_F32 = 0, 1, 2
UD_I64, UD_I32 = 0, 1
UD_TABLE_COHERENT, UD_TABLE_NONCOHERENT, UD_TABLE_PAD_ROWS = 0, 1, 2
UD_TUNE_NT_STORE, UD_TUNE_ELEMENTWISE = 2, 4
UD_TUNE_CIRCULAR_SHIFT, UD_TUNE_SHARE_GPU, UD_TUNE_DEST_ALIGNED, UD_TUNE_FLAT_SOURCE = 32, 128, 256, 512

#: every symbol include/ud.h declares
EXPORTS = (
    "ud_alloc_table", "ud_table_to_device", "ud_table_host_ptr", "ud_table_device_ptr",
    "ud_table_shape", "ud_table_pitch", "ud_free_table", "ud_gather", "ud_gather_noalloc", "ud_gather_pitched", "ud_gather_tuned", "ud_gather_plan",
    "ud_gather_status", "ud_cache_create", "ud_cache_free", "ud_gather_cached",
    "ud_scatter", "ud_scatter_tuned", "ud_scatter_pitched", "ud_status_str", "ud_last_hip_error", "ud_build_id",
)


class ud_tuning(ctypes.Structure):
    _fields_ = [
        ("lanes_per_row", ctypes.c_int32),
        ("chunks_per_lane", ctypes.c_int32),
        ("rows_in_flight", ctypes.c_int32),
        ("max_blocks", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
    ]


class UdError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        name = _lib.ud_status_str(status).decode()
        super().__init__(f"{where}: {name}" + (f" ({detail})" if detail else ""))


class UdIndexError(UdError):
    """A gather met an ID outside [0, N); ``pos`` is the smallest offending position."""

    def __init__(self, pos: int):
        self.pos = pos
        super().__init__(UD_ERR_INDEX_OUT_OF_RANGE, "ud_gather_status", f"position {pos}")


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build the HIP library first "
        "(python -m paper_2101_07956_amd.build). There is no fallback path."
    )

_lib = ctypes.CDLL(LIB_PATH)
_i64, _vp, _int = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int

_lib.ud_alloc_table.argtypes = [_i64, _i64, _int, ctypes.c_uint, ctypes.POINTER(_vp)]
_lib.ud_table_to_device.argtypes = [_vp, _i64, _i64, ctypes.POINTER(_vp)]
_lib.ud_table_host_ptr.argtypes = [_vp, ctypes.POINTER(_vp)]
_lib.ud_table_device_ptr.argtypes = [_vp, ctypes.POINTER(_vp)]
_lib.ud_table_shape.argtypes = [_vp, ctypes.POINTER(_i64), ctypes.POINTER(_i64), ctypes.POINTER(_int)]
_lib.ud_table_pitch.argtypes = [_vp, ctypes.POINTER(_i64)]
_lib.ud_gather_pitched.argtypes = [_vp, _i64, _i64, _i64, _int, _vp, _int, _i64, _vp, _vp]
_lib.ud_free_table.argtypes = [_vp]
_lib.ud_gather.argtypes = [_vp, _i64, _i64, _int, _vp, _int, _i64, _vp, _vp]
_lib.ud_gather_noalloc.argtypes = [_vp, _i64, _i64, _int, _vp, _int, _i64, _vp, _vp]
_lib.ud_gather_tuned.argtypes = [_vp, _i64, _i64, _int, _vp, _int, _i64, _vp, _vp, ctypes.POINTER(ud_tuning)]
_lib.ud_gather_plan.argtypes = [_vp, _i64, _int, ctypes.POINTER(ud_tuning)]
_lib.ud_gather_status.argtypes = [_vp, ctypes.POINTER(_i64)]
_lib.ud_scatter.argtypes = [_vp, _i64, _i64, _int, _vp, _int, _i64, _vp, _vp]
_lib.ud_scatter_pitched.argtypes = [_vp, _i64, _i64, _i64, _int, _vp, _int, _i64, _vp, _vp]
_lib.ud_scatter_tuned.argtypes = [_vp, _i64, _i64, _int, _vp, _int, _i64, _vp, _vp, ctypes.POINTER(ud_tuning)]
_lib.ud_cache_create.argtypes = [_vp, _vp, _i64, ctypes.POINTER(_vp)]
_lib.ud_cache_free.argtypes = [_vp]
_lib.ud_gather_cached.argtypes = [_vp, _int, _vp, _int, _i64, _vp, _vp]
_lib.ud_status_str.argtypes = [_int]
_lib.ud_status_str.restype = ctypes.c_char_p
_lib.ud_last_hip_error.argtypes = []
_lib.ud_last_hip_error.restype = ctypes.c_char_p
_lib.ud_build_id.argtypes = []
_lib.ud_build_id.restype = ctypes.c_char_p
for _n in EXPORTS[:-3]:
    getattr(_lib, _n).restype = _int


def _check(status: int, where: str) -> None:
    if status != UD_OK:
        detail = _lib.ud_last_hip_error().decode() if status in (UD_ERR_OOM, UD_ERR_HIP) else ""
        raise UdError(status, where, detail)


def ud_status_str(status: int) -> str:
    return _lib.ud_status_str(status).decode()


def ud_last_hip_error() -> str:
    return _lib.ud_last_hip_error().decode()


def ud_build_id() -> str:
    """Digest of the sources the loaded library was built from."""
    return _lib.ud_build_id().decode()


def ud_alloc_table(N: int, D: int, elem: int, flags: int = UD_TABLE_COHERENT) -> int:
    """Returns the opaque table handle (an integer address)."""
    t = _vp()
    _check(_lib.ud_alloc_table(N, D, elem, flags, ctypes.byref(t)), "ud_alloc_table")
    return t.value


def ud_table_to_device(src: int, row0: int, n: int) -> int:
    t = _vp()
    _check(_lib.ud_table_to_device(src, row0, n, ctypes.byref(t)), "ud_table_to_device")
    return t.value


def ud_table_host_ptr(t: int) -> int:
    p = _vp()
    _check(_lib.ud_table_host_ptr(t, ctypes.byref(p)), "ud_table_host_ptr")
    return p.value or 0


def ud_table_device_ptr(t: int) -> int:
    p = _vp()
    _check(_lib.ud_table_device_ptr(t, ctypes.byref(p)), "ud_table_device_ptr")
    return p.value or 0


def ud_table_shape(t: int) -> tuple[int, int, int]:
    N, D, e = _i64(), _i64(), _int()
    _check(_lib.ud_table_shape(t, ctypes.byref(N), ctypes.byref(D), ctypes.byref(e)), "ud_table_shape")
    return N.value, D.value, e.value


def ud_table_pitch(t: int) -> int:
    p = _i64()
    _check(_lib.ud_table_pitch(t, ctypes.byref(p)), "ud_table_pitch")
    return p.value


def ud_gather_pitched(table: int, N: int, D: int, pitch: int, dtype: int, idx: int, itype: int, M: int, out: int,
                      stream: int | None = None) -> None:
    """``ud_gather`` from a table whose rows are ``pitch`` elements apart."""
    _check(_lib.ud_gather_pitched(table, N, D, pitch, dtype, idx, itype, M, out, stream), "ud_gather_pitched")


def ud_free_table(t: int | None) -> None:
    _check(_lib.ud_free_table(t), "ud_free_table")


def ud_gather(table: int, N: int, D: int, dtype: int, idx: int, itype: int, M: int, out: int,
              stream: int | None = None) -> None:
    """Enqueue ``out[i, :] = conv(table[idx[i], :])``; all pointers are device addresses."""
    _check(_lib.ud_gather(table, N, D, dtype, idx, itype, M, out, stream), "ud_gather")


def ud_gather_noalloc(table: int, N: int, D: int, dtype: int, idx: int, itype: int, M: int, out: int,
                      stream: int | None = None) -> None:
    """``ud_gather`` for callers that must not allocate (static device error slots)."""
    _check(_lib.ud_gather_noalloc(table, N, D, dtype, idx, itype, M, out, stream), "ud_gather_noalloc")


def ud_gather_tuned(table: int, N: int, D: int, dtype: int, idx: int, itype: int, M: int, out: int,
                    stream: int | None = None, tuning: ud_tuning | None = None) -> None:
    ref = ctypes.byref(tuning) if tuning is not None else None
    _check(_lib.ud_gather_tuned(table, N, D, dtype, idx, itype, M, out, stream, ref), "ud_gather_tuned")


def ud_gather_plan(table: int, D: int, dtype: int) -> ud_tuning:
    plan = ud_tuning()
    _check(_lib.ud_gather_plan(table, D, dtype, ctypes.byref(plan)), "ud_gather_plan")
    return plan


def ud_gather_status(stream: int | None = None) -> None:
    """Waits for ``stream``; raises ``UdIndexError`` if a gather met a bad ID."""
    pos = _i64(-1)
    st = _lib.ud_gather_status(stream, ctypes.byref(pos))
    if st == UD_ERR_INDEX_OUT_OF_RANGE:
        raise UdIndexError(pos.value)
    _check(st, "ud_gather_status")


def ud_scatter(table: int, N: int, D: int, dtype: int, idx: int, itype: int, M: int, src: int,
               stream: int | None = None, tuning: ud_tuning | None = None) -> None:
    """Enqueue ``table[idx[i], :] = src[i, :]``; all pointers are device addresses."""
    if tuning is None:
        _check(_lib.ud_scatter(table, N, D, dtype, idx, itype, M, src, stream), "ud_scatter")
    else:
        _check(_lib.ud_scatter_tuned(table, N, D, dtype, idx, itype, M, src, stream, ctypes.byref(tuning)), "ud_scatter_tuned")


def ud_scatter_pitched(table: int, N: int, D: int, pitch: int, dtype: int, idx: int, itype: int, M: int, src: int,
                       stream: int | None = None) -> None:
    """``ud_scatter`` into a table whose rows are ``pitch`` elements apart."""
    _check(_lib.ud_scatter_pitched(table, N, D, pitch, dtype, idx, itype, M, src, stream), "ud_scatter_pitched")


def ud_cache_create(table: int, hot_rows_host_ptr: int, n_hot: int) -> int:
    """Hot-row cache over a host table; ``hot_rows_host_ptr`` is the CPU address of ``n_hot`` int64 row IDs."""
    c = _vp()
    _check(_lib.ud_cache_create(table, hot_rows_host_ptr, n_hot, ctypes.byref(c)), "ud_cache_create")
    return c.value


def ud_cache_free(c: int | None) -> None:
    _check(_lib.ud_cache_free(c), "ud_cache_free")


def ud_gather_cached(cache: int, dtype: int, idx: int, itype: int, M: int, out: int, stream: int | None = None) -> None:
    _check(_lib.ud_gather_cached(cache, dtype, idx, itype, M, out, stream), "ud_gather_cached")


def raw_status(fn_name: str, *args) -> int:
    """Call an exported function and return its bare status code (for error-path tests)."""
    return getattr(_lib, fn_name)(*args)
