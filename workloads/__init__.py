"""Seeded synthetic inputs (table fills, ID lists) shared by the oracle's tests
and the GPU library's tests and benchmark.

Input generation only: nothing of the gather lives here.  ``gen.c`` is built
with the host C compiler and OpenMP; values are pure functions of
(seed, flat element number), see that file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "gen.c"), os.path.join(_HERE, "graph.c")]
_LIB = os.path.join(_HERE, "libworkloads.so")


def build(force: bool = False) -> str:
    srcs = [s for s in _SRCS if os.path.exists(s)]
    stale = not os.path.exists(_LIB) or any(os.path.getmtime(_LIB) < os.path.getmtime(s) for s in srcs)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O3", "-std=gnu11", "-Wall", "-Wextra", "-fopenmp", "-fPIC", "-shared", *srcs,
             "-o", _LIB, "-lm"]
        )
    return _LIB


_lib = None
_u64 = ctypes.c_uint64
_vp = ctypes.c_void_p


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.wl_mix64.restype = _u64
        L.wl_mix64.argtypes = [_u64, _u64]
        L.wl_uniform_f32_at.restype = ctypes.c_float
        L.wl_uniform_f32_at.argtypes = [_u64, _u64]
        L.wl_normal_f16_at.restype = ctypes.c_uint16
        L.wl_normal_f16_at.argtypes = [_u64, _u64]
        L.wl_f32_to_f16_rne.restype = ctypes.c_uint16
        L.wl_f32_to_f16_rne.argtypes = [ctypes.c_float]
        for name in ("wl_fill_uniform_f32", "wl_fill_normal_f16"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [_vp, _u64, _u64, _u64]
        for name in ("wl_fill_tag_u32", "wl_fill_tag_u16"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [_vp, _u64, _u64]
        for name in ("wl_indices_uniform_i64", "wl_indices_uniform_i32"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [_vp, _u64, _u64, _u64]
        _lib = L
    return _lib


# ---- fills into caller memory (raw host address: numpy buffer or pinned table) ----

def fill_uniform_f32(ptr: int, seed: int, n: int, first: int = 0) -> None:
    """``n`` float32 values uniform in [-1, 1) written at host address ``ptr``."""
    lib().wl_fill_uniform_f32(ptr, seed, first, n)


def fill_normal_f16(ptr: int, seed: int, n: int, first: int = 0) -> None:
    """``n`` binary16 values, N(0,1) rounded to nearest even, at host address ``ptr``."""
    lib().wl_fill_normal_f16(ptr, seed, first, n)


def fill_tag(ptr: int, n: int, elem_bytes: int, first: int = 0) -> None:
    """Element e holds the integer e (mod 2**(8*elem_bytes)): closed-form expected gathers."""
    (lib().wl_fill_tag_u32 if elem_bytes == 4 else lib().wl_fill_tag_u16)(ptr, first, n)


# ---- numpy conveniences ----

def uniform_f32(seed: int, N: int, D: int) -> np.ndarray:
    a = np.empty((N, D), dtype=np.float32)
    fill_uniform_f32(a.ctypes.data, seed, N * D)
    return a


def normal_f16(seed: int, N: int, D: int) -> np.ndarray:
    a = np.empty((N, D), dtype=np.float16)
    fill_normal_f16(a.ctypes.data, seed, N * D)
    return a


def tag_table(N: int, D: int, elem_bytes: int = 4) -> np.ndarray:
    a = np.empty((N, D), dtype=np.uint32 if elem_bytes == 4 else np.uint16)
    fill_tag(a.ctypes.data, N * D, elem_bytes)
    return a


def indices_uniform(seed: int, M: int, N: int, dtype=np.int64) -> np.ndarray:
    """``M`` row IDs uniform in [0, N) with replacement."""
    a = np.empty(M, dtype=dtype)
    if np.dtype(dtype) == np.int64:
        lib().wl_indices_uniform_i64(a.ctypes.data, seed, M, N)
    elif np.dtype(dtype) == np.int32:
        assert N <= 2**31
        lib().wl_indices_uniform_i32(a.ctypes.data, seed, M, N)
    else:
        raise TypeError(dtype)
    return a


#: seed stream used for ID lists, kept apart from the table's value stream
IDX_STREAM = 0x1D5
