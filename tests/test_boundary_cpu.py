"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ud():
    import paper_2101_07956_amd as m
    return m


def test_library_exports_every_symbol_the_header_declares(ud):
    header = open(os.path.join(ROOT, "include", "ud.h")).read()
    declared = set(re.findall(r"\b(ud_[a-z_0-9]+)\s*\(", header))
    assert declared == set(ud.EXPORTS)
    lib = ctypes.CDLL(ud.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(ud):
    names = [ud.ud_status_str(s) for s in range(6)]
    assert names == ["UD_OK", "UD_ERR_INVALID_ARG", "UD_ERR_UNSUPPORTED", "UD_ERR_OOM",
                     "UD_ERR_INDEX_OUT_OF_RANGE", "UD_ERR_HIP"]
    assert ud.ud_status_str(99) == "UD_ERR_UNKNOWN"


def _gather(ud, table=0x1000, N=10, D=4, dtype=0, idx=0x2000, itype=0, M=5, out=0x3000, tuning=None):
    args = [table, N, D, dtype, idx, itype, M, out, None]
    if tuning is None:
        return ud.binding.raw_status("ud_gather", *args)
    return ud.binding.raw_status("ud_gather_tuned", *args, ctypes.byref(tuning))


def test_gather_rejects_bad_scalars_before_any_device_work(ud):
    inv = ud.UD_ERR_INVALID_ARG
    assert _gather(ud, N=0) == inv
    assert _gather(ud, N=-3) == inv
    assert _gather(ud, D=0) == inv
    assert _gather(ud, M=-1) == inv
    assert _gather(ud, dtype=3) == inv
    assert _gather(ud, dtype=-1) == inv
    assert _gather(ud, itype=2) == inv
    assert _gather(ud, table=None) == inv
    assert _gather(ud, idx=None) == inv
    assert _gather(ud, out=None) == inv
    assert _gather(ud, table=0x1002) == inv            # fp32 table must be 4-byte aligned
    assert _gather(ud, table=0x1001, dtype=1) == inv   # fp16 table must be 2-byte aligned
    assert _gather(ud, out=0x3002) == inv
    assert _gather(ud, idx=0x2004) == inv              # int64 IDs must be 8-byte aligned
    assert _gather(ud, N=2**40, D=2**30) == inv        # byte count overflows int64
    assert _gather(ud, M=2**40, D=2**30, N=4) == inv


def test_scatter_rejects_bad_arguments(ud):
    inv = ud.UD_ERR_INVALID_ARG
    rs = ud.binding.raw_status
    ok_args = [0x1000, 10, 4, 0, 0x2000, 0, 5, 0x3000, None]
    for pos, val in ((1, 0), (2, 0), (6, -1), (3, 2), (3, 7), (5, 3), (0, None), (4, None), (7, None), (0, 0x1002), (7, 0x3001)):
        a = list(ok_args)
        a[pos] = val
        assert rs("ud_scatter", *a) == inv, (pos, val)
    a = list(ok_args)
    a[6] = 0
    assert rs("ud_scatter", *a) == ud.UD_OK                 # M == 0: no-op, no device needed
    T = ud.ud_tuning
    for tun, want in ((T(0, 0, 0, 0, ud.UD_TUNE_FLAT_SOURCE), ud.UD_OK), (T(0, 3, 0, 0, ud.UD_TUNE_FLAT_SOURCE), ud.UD_ERR_UNSUPPORTED),
                      (T(0, 0, 0, 0, ud.UD_TUNE_NT_STORE), inv), (T(3, 0, 0, 0, 0), inv),
                      (T(0, 0, 0, 0, ud.UD_TUNE_FLAT_SOURCE | ud.UD_TUNE_NT_STORE), ud.UD_OK)):
        assert rs("ud_scatter_tuned", *a, ctypes.byref(tun)) == want


def test_empty_gather_is_ok_without_a_device(ud):
    assert _gather(ud, M=0, table=None, idx=None, out=None) == ud.UD_OK


def test_tuning_fields_are_range_checked(ud):
    T = ud.ud_tuning
    inv = ud.UD_ERR_INVALID_ARG
    assert _gather(ud, tuning=T(3, 0, 0, 0, 0)) == inv       # not a power of two
    assert _gather(ud, tuning=T(128, 0, 0, 0, 0)) == inv
    assert _gather(ud, tuning=T(0, 5, 0, 0, 0)) == inv
    assert _gather(ud, tuning=T(0, 0, 3, 0, 0)) == inv
    assert _gather(ud, tuning=T(0, 0, 0, -1, 0)) == inv
    assert _gather(ud, tuning=T(0, 0, 0, 0, 512)) == inv      # unknown flag
    for gone in (1, 8, 16, 64):                                 # options earlier versions had: no longer accepted
        assert _gather(ud, tuning=T(0, 0, 0, 0, gone)) == inv
    assert _gather(ud, tuning=T(0, 0, 0, 0, 32)) == inv       # circular shift needs the one-lane-per-element kernel
    DA = ud.UD_TUNE_DEST_ALIGNED
    for other in (ud.UD_TUNE_ELEMENTWISE, ud.UD_TUNE_SHARE_GPU):
        assert _gather(ud, tuning=T(0, 0, 0, 0, DA | other)) == inv
    assert _gather(ud, tuning=T(0, 3, 0, 0, DA)) == ud.UD_ERR_UNSUPPORTED     # 1, 2 or 4 output chunks per lane
    assert _gather(ud, M=0, tuning=T(0, 4, 0, 0, DA | ud.UD_TUNE_NT_STORE)) == ud.UD_OK
    assert _gather(ud, M=0, D=2**31, N=1, tuning=T(0, 1, 0, 0, DA)) == ud.UD_ERR_UNSUPPORTED   # columns are 32-bit there
    assert _gather(ud, tuning=T(0, 0, 8, 0, 0)) == inv
    assert _gather(ud, tuning=T(0, 4, 4, 0, 0)) == ud.UD_ERR_UNSUPPORTED   # no such instantiation
    assert _gather(ud, tuning=T(0, 2, 4, 0, 0)) == ud.UD_ERR_UNSUPPORTED
    assert _gather(ud, M=0, tuning=T(64, 2, 2, 0, 2)) == ud.UD_OK


def test_table_calls_reject_bad_arguments(ud):
    inv = ud.UD_ERR_INVALID_ARG
    t = ctypes.c_void_p()
    rs = ud.binding.raw_status
    assert rs("ud_alloc_table", 0, 4, 0, 0, ctypes.byref(t)) == inv
    assert rs("ud_alloc_table", 4, 0, 0, 0, ctypes.byref(t)) == inv
    assert rs("ud_alloc_table", 4, 4, 2, 0, ctypes.byref(t)) == inv      # UD_F16_TO_F32 is not a storage type
    assert rs("ud_alloc_table", 4, 4, 0, 4, ctypes.byref(t)) == inv      # unknown flag
    assert rs("ud_table_pitch", None, None) == inv
    assert rs("ud_gather_pitched", 0x1000, 4, 8, 7, 0, 0x2000, 0, 1, 0x3000, None) == inv   # pitch < D
    assert rs("ud_alloc_table", 4, 4, 0, 0, None) == inv
    assert rs("ud_alloc_table", 2**40, 2**30, 0, 0, ctypes.byref(t)) == inv
    assert rs("ud_table_to_device", None, 0, 1, ctypes.byref(t)) == inv
    assert rs("ud_table_host_ptr", None, ctypes.byref(t)) == inv
    assert rs("ud_table_device_ptr", None, ctypes.byref(t)) == inv
    assert rs("ud_table_shape", None, None, None, None) == inv
    assert rs("ud_free_table", None) == ud.UD_OK                          # NULL is a no-op
    assert rs("ud_cache_create", None, None, 1, ctypes.byref(t)) == inv
    assert rs("ud_gather_cached", None, 0, 0x1000, 0, 1, 0x2000, None) == inv
    assert rs("ud_cache_free", None) == ud.UD_OK


def test_plan_follows_row_width(ud):
    # an address the runtime does not know counts as host memory: one row per wavefront
    # instruction for rows longer than 64 bytes, natural group size below
    for D, lanes, chunks in [(16, 4, 1), (24, 64, 1), (32, 64, 1), (64, 64, 1), (100, 64, 1), (128, 64, 1), (256, 64, 1),
                             (602, 64, 3), (4096, 64, 4)]:
        p = ud.ud_gather_plan(0x10000, D, ud.UD_F32)
        assert (p.lanes_per_row, p.chunks_per_lane) == (lanes, chunks), D
        assert p.rows_in_flight * p.chunks_per_lane <= 8
    p = ud.ud_gather_plan(0x10000, 602, ud.UD_F16_TO_F32)
    assert (p.lanes_per_row, p.chunks_per_lane) == (64, 2)
    # rows that start at 4 different offsets modulo 16 can overlap one more chunk
    p = ud.ud_gather_plan(0x10000, 255, ud.UD_F32)      # 1020-byte rows: up to 65 chunks
    assert (p.lanes_per_row, p.chunks_per_lane) == (64, 2)


def test_build_stamp_matches_the_sources(ud):
    # the library says which sources it was built from; the build module recognises a stale one
    from paper_2101_07956_amd import build
    assert not build.stale()
    assert ud.ud_build_id() == build.source_digest()


def test_header_is_plain_c_and_the_library_links_from_c(ud, tmp_path):
    import subprocess
    exe = str(tmp_path / "c_abi_check")
    pkg = os.path.dirname(ud.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                           "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c_abi_check.c"),
                           "-o", exe, "-L", pkg, "-lud", "-Wl,-rpath," + pkg])
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0 and "c abi ok" in r.stdout, (r.returncode, r.stdout, r.stderr)


def test_environment_override_reaches_ud_gather():
    # UD_GATHER_TUNING makes ud_gather validate (and use) explicit kernel parameters: an unsupported
    # combination is refused, where the same call without the variable is accepted
    import subprocess
    import sys
    code = ("import sys; sys.path.insert(0, %r)\n"
            "import paper_2101_07956_amd as ud\n"
            "print(ud.binding.raw_status('ud_gather', 0x1000, 10, 4, 0, 0x2000, 0, 0, 0x3000, None))\n" % ROOT)
    plain = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env={**os.environ})
    forced = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True,
                            env={**os.environ, "UD_GATHER_TUNING": "64,4,4,0,0"})
    garbage = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True,
                             env={**os.environ, "UD_GATHER_TUNING": "fast please"})
    assert plain.stdout.strip() == "0" and forced.stdout.strip() == "2" and garbage.stdout.strip() == "0"
