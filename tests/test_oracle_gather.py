"""Pins for the CPU oracle's gather (no GPU).

The oracle is the definition out[i, :] = table[idx[i], :] (PyTorch-Direct,
Section 2.2 and Listings 1-2).  It is pinned here against things that are not
the oracle: an exhaustive literal enumeration on tiny shapes, numpy's take,
closed-form "tag" tables whose expected output needs no table at all, and the
invariants a gather must have.
"""
import itertools

import numpy as np
import pytest

import oracle
import workloads


def test_brute_force_every_index_tuple_on_tiny_shapes():
    # every (N, D, M) with N<=4, D<=3, M<=3 and every idx tuple in [0,N)^M
    rng = np.random.default_rng(7)
    for N, D, M in itertools.product(range(1, 5), range(1, 4), range(0, 4)):
        rows = [[int(rng.integers(0, 2**32)) for _ in range(D)] for _ in range(N)]
        table = np.array(rows, dtype=np.uint32).reshape(N, D)
        for tup in itertools.product(range(N), repeat=M):
            got = oracle.gather(table, np.array(tup, dtype=np.int64))
            assert got.shape == (M, D)
            want = [[rows[r][c] for c in range(D)] for r in tup]   # plain lists, no arrays
            assert got.tolist() == want


@pytest.mark.parametrize("D", [1, 3, 16, 100, 128, 602, 603])
@pytest.mark.parametrize("idt", [np.int64, np.int32])
def test_matches_numpy_take(D, idt):
    N, M = 997, 2311
    table = workloads.uniform_f32(11, N, D)
    idx = workloads.indices_uniform(12, M, N, idt)
    got = oracle.gather(table, idx)
    want = np.take(table, idx, axis=0)
    assert got.dtype == np.float32
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("N,D", [(50, 7), (333, 100), (4099, 602)])
def test_tag_table_closed_form(N, D):
    # element (r, c) holds r*D + c, so out[i, j] must be idx[i]*D + j
    table = workloads.tag_table(N, D)
    idx = workloads.indices_uniform(3, 1000, N)
    got = oracle.gather(table, idx).astype(np.int64)
    want = idx[:, None] * D + np.arange(D)[None, :]
    assert np.array_equal(got, want)


def test_tag_table_closed_form_2byte():
    N, D = 100, 13          # N*D < 65536 so tags are unique
    table = workloads.tag_table(N, D, elem_bytes=2)
    idx = workloads.indices_uniform(4, 500, N, np.int32)
    got = oracle.gather(table, idx).astype(np.int64)
    assert got.shape == (500, D)
    assert np.array_equal(got, idx.astype(np.int64)[:, None] * D + np.arange(D)[None, :])


def test_arange_is_identity_and_slices():
    table = workloads.uniform_f32(5, 321, 37)
    assert oracle.gather(table, np.arange(321)).tobytes() == table.tobytes()
    assert oracle.gather(table, np.arange(17, 200)).tobytes() == table[17:200].tobytes()
    assert oracle.gather(table, np.arange(320, -1, -1)).tobytes() == table[::-1].tobytes()


def test_constant_and_last_row_index():
    table = workloads.uniform_f32(6, 64, 9)
    out = oracle.gather(table, np.full(40, 63, dtype=np.int64))
    assert (out == table[63]).all() and out.shape == (40, 9)
    out = oracle.gather(table, np.zeros(5, dtype=np.int32))
    assert (out == table[0]).all()


def test_repeated_indices_give_identical_rows():
    table = workloads.uniform_f32(8, 500, 33)
    idx = workloads.indices_uniform(9, 4000, 500)          # many repeats
    out = oracle.gather(table, idx)
    order = np.argsort(idx, kind="stable")
    same = idx[order][1:] == idx[order][:-1]
    a, b = out[order][1:][same], out[order][:-1][same]
    assert same.sum() > 1000 and np.array_equal(a, b)


def test_permuting_indices_permutes_rows():
    table = workloads.uniform_f32(10, 700, 21)
    idx = workloads.indices_uniform(11, 1234, 700)
    perm = np.random.default_rng(1).permutation(idx.size)
    assert np.array_equal(oracle.gather(table, idx[perm]), oracle.gather(table, idx)[perm])


def test_bit_patterns_survive_unchanged():
    # NaNs with payloads, -0, infinities, subnormals: copied as bits, not as floats
    pats = np.array([0x7fc00001, 0xffc12345, 0x7f800001, 0x80000000, 0x00000001,
                     0x7f800000, 0xff800000, 0x807fffff], dtype=np.uint32)
    table = np.stack([pats, pats[::-1]]).view(np.float32)
    out = oracle.gather(table, np.array([1, 0, 1]))
    assert out.view(np.uint32).tolist() == [pats[::-1].tolist(), pats.tolist(), pats[::-1].tolist()]
    h = np.arange(0x7c00, 0x7c10, dtype=np.uint16).reshape(2, 8)
    assert oracle.gather(h, np.array([1, 1, 0]), oracle.F16).tolist() == [h[1].tolist(), h[1].tolist(), h[0].tolist()]


def test_empty_index_list():
    table = workloads.uniform_f32(1, 10, 4)
    out = oracle.gather(table, np.empty(0, dtype=np.int64))
    assert out.shape == (0, 4)


@pytest.mark.parametrize("idt", [np.int64, np.int32])
@pytest.mark.parametrize("bad", [-1, 50, 51, 2**31 - 1, -2**31])
def test_out_of_range_is_rejected_with_first_position_and_nothing_written(idt, bad):
    N, D = 50, 6
    table = workloads.uniform_f32(2, N, D)
    idx = np.arange(40, dtype=idt) % N
    idx[17] = bad
    idx[29] = bad          # a later bad entry must not be the one reported
    out = np.full((40, D), 0xA5A5A5A5, dtype=np.uint32)
    with pytest.raises(oracle.OracleIndexError) as e:
        oracle.gather_raw(table.ctypes.data, N, D, oracle.F32, idx, out)
    assert e.value.pos == 17
    assert (out == 0xA5A5A5A5).all()
    idx[17] = N - 1        # largest valid id is accepted
    idx[29] = 0
    oracle.gather_raw(table.ctypes.data, N, D, oracle.F32, idx, out)
    assert np.array_equal(out[17], table[N - 1].view(np.uint32))


def test_int64_index_beyond_32_bits_is_rejected():
    table = workloads.uniform_f32(2, 8, 2)
    with pytest.raises(oracle.OracleIndexError) as e:
        oracle.gather(table, np.array([1, 2**32 + 1], dtype=np.int64))   # would alias row 1 if truncated
    assert e.value.pos == 1


def test_writes_exactly_m_times_d_elements():
    N, D, M = 30, 5, 12
    table = workloads.uniform_f32(3, N, D)
    buf = np.full(M * D + 64, 0xDEADBEEF, dtype=np.uint32)
    out = buf[:M * D].reshape(M, D)
    oracle.gather_raw(table.ctypes.data, N, D, oracle.F32, workloads.indices_uniform(1, M, N), out)
    assert (buf[M * D:] == 0xDEADBEEF).all()
    assert not (out == 0xDEADBEEF).any()


def test_invalid_arguments():
    table = workloads.uniform_f32(3, 4, 4)
    out = np.empty((1, 4), dtype=np.uint32)
    idx = np.zeros(1, dtype=np.int64)
    for N, D in [(0, 4), (4, 0), (-1, 4)]:
        with pytest.raises(ValueError):
            oracle.gather_raw(table.ctypes.data, N, D, oracle.F32, idx, out)
    with pytest.raises(ValueError):
        oracle.gather_raw(table.ctypes.data, 4, 4, 7, idx, out)


@pytest.mark.parametrize("D,pitch", [(1, 1), (3, 8), (100, 128), (602, 608), (602, 602), (5, 37)])
def test_pitched_table_matches_numpy_on_the_padded_array(D, pitch):
    # rows `pitch` elements apart, only the first D of each are data
    N, M = 501, 777
    padded = workloads.uniform_f32(21, N, pitch)
    idx = workloads.indices_uniform(22, M, N)
    out = np.full((M, D), 0xA5A5A5A5, dtype=np.uint32)
    oracle.gather_raw(padded.ctypes.data, N, D, oracle.F32, idx, out, pitch=pitch)
    assert np.array_equal(out, np.take(padded, idx, axis=0)[:, :D].view(np.uint32))


def test_pitched_tag_table_closed_form_and_padding_is_never_read():
    N, D, pitch, M = 300, 11, 16, 400
    table = workloads.tag_table(N, pitch)                       # element (r, c) of the padded array holds r*pitch + c
    table[:, D:] = 0xFFFFFFFF                                    # poison the padding
    idx = workloads.indices_uniform(23, M, N, np.int32)
    out = np.empty((M, D), dtype=np.uint32)
    oracle.gather_raw(table.ctypes.data, N, D, oracle.F32, idx, out, pitch=pitch)
    assert np.array_equal(out.astype(np.int64), idx.astype(np.int64)[:, None] * pitch + np.arange(D)[None, :])


def test_pitch_smaller_than_width_is_invalid():
    table = workloads.uniform_f32(24, 4, 8)
    with pytest.raises(ValueError):
        oracle.gather_raw(table.ctypes.data, 4, 8, oracle.F32, np.zeros(1, dtype=np.int64),
                          np.empty((1, 8), dtype=np.uint32), pitch=7)
