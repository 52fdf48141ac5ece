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
        _i64 = ctypes.c_int64
        _dbl = ctypes.c_double
        L.wl_node_of_rank.restype = _i64
        L.wl_node_of_rank.argtypes = [_u64, _u64, _u64]
        L.wl_nodes_of_ranks.restype = None
        L.wl_nodes_of_ranks.argtypes = [_vp, _u64, _u64, _u64, _u64]
        L.wl_zipf_rank.restype = _u64
        L.wl_zipf_rank.argtypes = [_u64, _u64, _u64, _dbl]
        L.wl_graph_degrees.restype = _i64
        L.wl_graph_degrees.argtypes = [_vp, _u64, _dbl, _i64, _u64]
        L.wl_graph_fill_ids.restype = None
        L.wl_graph_fill_ids.argtypes = [_vp, _vp, _u64, _dbl, _u64]
        L.wl_sample_csr.restype = _i64
        L.wl_sample_csr.argtypes = [_vp, _vp, _u64, _i64, _vp, ctypes.c_int, _u64, _u64, _vp, _i64]
        L.wl_sample_procedural.restype = _i64
        L.wl_sample_procedural.argtypes = [_u64, _i64, _dbl, _u64, _i64, _vp, ctypes.c_int, _u64, _u64, _vp, _i64]
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


# ---- power-law graphs and minibatch neighbour sampling (see graph.c) ----

def zipf_graph_csr(N: int, mean_degree: float, dmin: int, alpha: float, seed: int):
    """CSR (int64 offsets[N+1], int64 ids[E]) of a Zipf(1.0)-degree graph with degree floor ``dmin``
    and neighbour popularity ~ rank**-alpha."""
    deg = np.empty(N, dtype=np.int64)
    total = lib().wl_graph_degrees(deg.ctypes.data, N, float(mean_degree), dmin, seed)
    offsets = np.zeros(N + 1, dtype=np.int64)
    np.cumsum(deg, out=offsets[1:])
    assert offsets[-1] == total
    ids = np.empty(total, dtype=np.int64)
    lib().wl_graph_fill_ids(offsets.ctypes.data, ids.ctypes.data, N, float(alpha), seed)
    return offsets, ids


def hottest_nodes(N: int, n: int, graph_seed: int) -> np.ndarray:
    """The ``n`` most popular nodes of a graph built with ``graph_seed`` (popularity ranks 1..n)."""
    out = np.empty(n, dtype=np.int64)
    lib().wl_nodes_of_ranks(out.ctypes.data, 1, n, N, graph_seed)
    return out


def slot_bound(nseeds: int, fanout) -> int:
    n = nseeds
    for f in fanout:
        n *= 1 + f
    return n


def sample_csr(offsets: np.ndarray, ids: np.ndarray, nseeds: int, fanout, seed: int, batch: int) -> np.ndarray:
    """Distinct node IDs of one minibatch, first-occurrence order, seeds first."""
    fan = np.asarray(fanout, dtype=np.int64)
    cap = slot_bound(nseeds, fanout)
    out = np.empty(cap, dtype=np.int64)
    n = lib().wl_sample_csr(offsets.ctypes.data, ids.ctypes.data, offsets.size - 1, nseeds, fan.ctypes.data,
                            fan.size, seed, batch, out.ctypes.data, cap)
    if n < 0:
        raise MemoryError("wl_sample_csr failed")
    return out[:n].copy()


def sample_procedural(N: int, degree: int, alpha: float, graph_seed: int, nseeds: int, fanout, seed: int,
                      batch: int) -> np.ndarray:
    """Same for the never-materialised graph in which every node has ``degree`` hashed neighbour slots."""
    fan = np.asarray(fanout, dtype=np.int64)
    cap = slot_bound(nseeds, fanout)
    out = np.empty(cap, dtype=np.int64)
    n = lib().wl_sample_procedural(N, degree, float(alpha), graph_seed, nseeds, fan.ctypes.data, fan.size, seed,
                                   batch, out.ctypes.data, cap)
    if n < 0:
        raise MemoryError("wl_sample_procedural failed")
    return out[:n].copy()


#: the two GraphSAGE-style workloads: graph and sampling parameters.  alpha (neighbour popularity ~ rank**-alpha)
#: is set so that a de-duplicated minibatch holds about 200K (products-like) and 500K (papers-like) IDs; with
#: alpha = 1.0 the batches would be several times smaller
PRODUCTS_LIKE = dict(N=2_400_000, D=100, mean_degree=50, dmin=25, alpha=0.6, nseeds=1024, fanout=(25, 10))
PAPERS_LIKE = dict(N=111_000_000, D=256, degree=30, alpha=0.8, nseeds=1024, fanout=(15, 10, 5))
