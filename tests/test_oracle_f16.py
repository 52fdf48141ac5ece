"""Pins for the oracle's binary16 -> binary32 widening (no GPU).

Checked against: textbook encodings (tests/golden/binary16_values.txt), numpy's
float16 -> float32 cast on every non-NaN pattern, the x86 F16C hardware
converter on all 65,536 patterns (NaNs included), exact round trip, and
order preservation.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
ALL = np.arange(65536, dtype=np.uint32).astype(np.uint16)
IS_NAN = ((ALL & 0x7c00) == 0x7c00) & ((ALL & 0x03ff) != 0)


@pytest.fixture(scope="module")
def widened():
    return oracle.f16_bits_to_f32_bits(ALL)


def test_textbook_values(widened):
    n = 0
    for line in open(os.path.join(HERE, "golden", "binary16_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        h, f = line.split()[:2]
        assert int(widened[int(h, 16)]) == int(f, 16), line
        n += 1
    assert n >= 20


def test_all_non_nan_patterns_match_numpy_cast(widened):
    want = ALL.view(np.float16).astype(np.float32).view(np.uint32)
    assert IS_NAN.sum() == 2046
    assert np.array_equal(widened[~IS_NAN], want[~IS_NAN])


def test_nan_patterns_keep_sign_and_payload_and_come_out_quiet(widened):
    w = widened[IS_NAN]
    h = ALL[IS_NAN].astype(np.uint32)
    assert ((w >> 31) == (h >> 15)).all()
    assert (((w >> 23) & 0xff) == 0xff).all()
    assert ((w & 0x00400000) != 0).all()                         # quiet bit
    assert (((w >> 13) & 0x1ff) == (h & 0x1ff)).all()            # low 9 payload bits in place
    assert ((w & 0x1fff) == 0).all()
    assert np.isnan(w.view(np.float32)).all()


def _f16c():
    if "f16c" not in open("/proc/cpuinfo").read():
        pytest.skip("CPU has no F16C")
    so = os.path.join(HERE, "_f16c_helper.so")
    src = os.path.join(HERE, "f16c_helper.c")
    if not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O1", "-mf16c", "-fPIC", "-shared", src, "-o", so])
    lib = ctypes.CDLL(so)
    lib.f16c_widen.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
    lib.f16c_widen.restype = None
    return lib


def test_all_65536_patterns_match_the_f16c_hardware_converter(widened):
    lib = _f16c()
    hw = np.empty(65536, dtype=np.uint32)
    lib.f16c_widen(ALL.ctypes.data, hw.ctypes.data, 65536)
    assert np.array_equal(widened, hw)


def test_round_trip_is_exact(widened):
    back = widened.view(np.float32)[~IS_NAN].astype(np.float16).view(np.uint16)
    assert np.array_equal(back, ALL[~IS_NAN])


def test_order_is_preserved(widened):
    pos = widened[0:0x7c01].view(np.float32)          # +0 ... +inf
    assert (np.diff(pos.astype(np.float64)) > 0).all()
    neg = widened[0x8000:0xfc01].view(np.float32)     # -0 ... -inf
    assert (np.diff(neg.astype(np.float64)) < 0).all()


def test_widening_gather_uses_the_same_conversion(widened):
    table = ALL.reshape(256, 256)
    idx = np.random.default_rng(0).permutation(256)
    out = oracle.gather(table, idx, oracle.F16_TO_F32)
    assert out.dtype == np.float32 and out.shape == (256, 256)
    assert np.array_equal(out.view(np.uint32), widened.reshape(256, 256)[idx])
