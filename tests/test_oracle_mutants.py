"""Do the pins bite?  Plausible mistakes are planted in copies of the oracle's C source (on the CPU only);
each mutant must fail at least one of the independent checks the pin tests are made of, and the
unmodified source must pass them all."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "gather_oracle.c")

MUTANTS = {
    "transposed source index": ("const int64_t src = r * pitch + j;", "const int64_t src = r + j * N;"),
    "source row off by one": ("const int64_t src = r * pitch + j;", "const int64_t src = (r + 1 < N ? r + 1 : r) * pitch + j;"),
    "destination uses the ID": ("const int64_t dst = i * D + j;", "const int64_t dst = (r % M) * D + j;"),
    "last column dropped": ("for (int64_t j = 0; j < D; ++j) {\n            const int64_t src", "for (int64_t j = 0; j + 1 < D || j == 0; ++j) {\n            const int64_t src"),
    "upper bound off by one": ("if (r < 0 || r >= N) {\n            if (bad_pos)\n                *bad_pos = i;\n            return ORACLE_ERR_INDEX;", "if (r < 0 || r > N) {\n            if (bad_pos)\n                *bad_pos = i;\n            return ORACLE_ERR_INDEX;"),
    "negative IDs wrapped": ("if (r < 0 || r >= N) {\n            if (bad_pos)\n                *bad_pos = i;\n            return ORACLE_ERR_INDEX;", "if (r < -N || r >= N) {\n            if (bad_pos)\n                *bad_pos = i;\n            return ORACLE_ERR_INDEX;"),
    "int32 IDs read as int64": ("return (int64_t)((const int32_t *)idx)[i];", "return ((const int64_t *)idx)[i / 2] & 0xffffffff;"),
    "half exponent bias wrong": ("v = ldexp((double)(1024u + f), (int)e - 25);", "v = ldexp((double)(1024u + f), (int)e - 24);"),
    "subnormals flushed": ("v = ldexp((double)f, -24);", "v = 0.0;"),
    "sign of zero lost": ("return bits | (s << 31);                           /* sign last, so -0 survives */", "return (bits ? bits | (s << 31) : 0);"),
    "NaN not quieted": ("bits = 0x7f800000u | 0x00400000u | (f << 13);", "bits = 0x7f800000u | (f << 13);"),
    "NaN payload dropped": ("bits = 0x7f800000u | 0x00400000u | (f << 13);", "bits = 0x7fc00000u;"),
    "scatter writes the wrong row": ("((uint32_t *)table)[r * pitch + j] = ((const uint32_t *)src)[i * D + j];", "((uint32_t *)table)[i * pitch + j] = ((const uint32_t *)src)[i * D + j];"),
    "shift sign flipped": ("int64_t s = ((i - r) * D) % elems_per_line;", "int64_t s = ((r - i) * D) % elems_per_line;"),
    "request model counts lines only": ("seen = (warp[b] == warp[a] && line[b] == line[a]);", "seen = (line[b] == line[a]);"),
}


def build(source_text, path):
    c = path + ".c"
    open(c, "w").write(source_text)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", c, "-o", path, "-lm"])
    lib = ctypes.CDLL(path)
    lib.oracle_f16_bits_to_f32_bits.restype = ctypes.c_uint32
    lib.oracle_f16_bits_to_f32_bits.argtypes = [ctypes.c_uint16]
    i64, vp = ctypes.c_int64, ctypes.c_void_p
    lib.oracle_gather.argtypes = [vp, i64, i64, ctypes.c_int, vp, ctypes.c_int, i64, vp, ctypes.POINTER(i64)]
    lib.oracle_scatter.argtypes = [vp, i64, i64, ctypes.c_int, vp, ctypes.c_int, i64, vp, ctypes.POINTER(i64)]
    lib.oracle_count_requests.restype = i64
    lib.oracle_count_requests.argtypes = [vp, vp, i64, i64, i64, i64, i64, i64, i64]
    lib.oracle_circular_shift.restype = i64
    lib.oracle_circular_shift.argtypes = [i64] * 4
    return lib


def pins_pass(lib) -> bool:
    """A compact version of the pin tests, against an arbitrary build of the oracle."""
    rng = np.random.default_rng(5)
    bad = ctypes.c_int64()

    def gather(table, idx, dtype=0):
        out = np.zeros((idx.size, table.shape[1]), dtype=np.uint32 if dtype != 1 else np.uint16)
        rc = lib.oracle_gather(table.ctypes.data, table.shape[0], table.shape[1], dtype, idx.ctypes.data,
                               0 if idx.dtype == np.int64 else 1, idx.size, out.ctypes.data, ctypes.byref(bad))
        return rc, out

    # gather: numpy.take, tag closed form, both ID types, last row, bounds
    for N, D, M in ((7, 3, 11), (40, 5, 64), (300, 17, 200)):
        table = rng.integers(0, 2**32, size=(N, D), dtype=np.uint64).astype(np.uint32)
        for idt in (np.int64, np.int32):
            idx = rng.integers(0, N, size=M).astype(idt)
            idx[0] = N - 1
            rc, out = gather(table, idx)
            if rc != 0 or not np.array_equal(out, np.take(table, idx, axis=0)):
                return False
        tag = np.arange(N * D, dtype=np.uint32).reshape(N, D)
        rc, out = gather(tag, idx.astype(np.int64))
        if not np.array_equal(out.astype(np.int64), idx.astype(np.int64)[:, None] * D + np.arange(D)):
            return False
        for value, ok in ((N, False), (-1, False), (N - 1, True)):
            probe = np.array([0, value], dtype=np.int64)
            rc, _ = gather(table, probe)
            if (rc == 0) != ok or (not ok and bad.value != 1):
                return False
    # scatter: numpy assignment
    table = rng.integers(0, 2**32, size=(50, 4), dtype=np.uint64).astype(np.uint32)
    want = table.copy()
    idx = rng.permutation(50)[:20].astype(np.int64)
    src = rng.integers(0, 2**32, size=(20, 4), dtype=np.uint64).astype(np.uint32)
    lib.oracle_scatter(table.ctypes.data, 50, 4, 0, idx.ctypes.data, 0, 20, src.ctypes.data, ctypes.byref(bad))
    want[idx] = src
    if not np.array_equal(table, want):
        return False
    # widening: numpy on every non-NaN pattern, the bit rule on NaNs
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = np.array([lib.oracle_f16_bits_to_f32_bits(int(x)) for x in h], dtype=np.uint32)
    nan = ((h & 0x7c00) == 0x7c00) & ((h & 0x3ff) != 0)
    if not np.array_equal(got[~nan], h.view(np.float16).astype(np.float32).view(np.uint32)[~nan]):
        return False
    hn = h[nan].astype(np.uint32)
    if not np.array_equal(got[nan], ((hn & 0x8000) << 16) | 0x7fc00000 | ((hn & 0x3ff) << 13)):
        return False
    # request model: the paper's 7 -> 5 with a shift of 1
    rows = np.array([0, 2, 4], dtype=np.int64)
    if lib.oracle_count_requests(rows.ctypes.data, None, 3, 11, 4, 4, 16, 1, 2) != 7:
        return False
    s = np.array([lib.oracle_circular_shift(i, int(r), 11, 4) for i, r in enumerate(rows)], dtype=np.int64)
    return s[1] == 1 and lib.oracle_count_requests(rows.ctypes.data, s.ctypes.data, 3, 11, 4, 4, 16, 1, 2) == 5


def test_the_real_oracle_passes(tmp_path):
    assert pins_pass(build(open(SRC).read(), str(tmp_path / "liboracle_ref.so")))


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_every_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name!r} not found: update the mutant table"
    lib = build(text.replace(old, new), str(tmp_path / "liboracle_mutant.so"))
    assert not pins_pass(lib), f"no pin noticed: {name}"
