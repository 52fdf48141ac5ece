"""Pins for the oracle's write direction, table[idx[i], :] = src[i, :] (no GPU)."""
import itertools

import numpy as np
import pytest

import oracle
import workloads


def test_brute_force_every_index_tuple_on_tiny_shapes():
    rng = np.random.default_rng(3)
    for N, D, M in itertools.product(range(1, 5), range(1, 4), range(0, 4)):
        base = [[int(rng.integers(0, 2**32)) for _ in range(D)] for _ in range(N)]
        src = [[int(rng.integers(0, 2**32)) for _ in range(D)] for _ in range(M)]
        for tup in itertools.product(range(N), repeat=M):
            table = np.array(base, dtype=np.uint32).reshape(N, D)
            oracle.scatter(table, np.array(tup, dtype=np.int64), np.array(src, dtype=np.uint32).reshape(M, D))
            want = [row[:] for row in base]              # plain lists: apply the writes in order
            for i, r in enumerate(tup):
                for c in range(D):
                    want[r][c] = src[i][c]
            assert table.tolist() == want


@pytest.mark.parametrize("D", [1, 3, 100, 602])
@pytest.mark.parametrize("idt", [np.int64, np.int32])
def test_matches_numpy_fancy_assignment(D, idt):
    N, M = 1000, 700
    table = workloads.uniform_f32(1, N, D)
    want = table.copy()
    idx = workloads.indices_uniform(2, M, N, idt)          # has duplicates: numpy keeps the last, like the oracle
    src = workloads.uniform_f32(3, M, D)
    oracle.scatter(table, idx, src)
    want[idx] = src
    assert np.array_equal(table.view(np.uint32), want.view(np.uint32))


def test_scatter_then_gather_returns_the_source_and_other_rows_are_untouched():
    N, D, M = 5000, 37, 1200
    table = workloads.uniform_f32(4, N, D)
    before = table.copy()
    idx = np.random.default_rng(5).permutation(N)[:M].astype(np.int64)     # distinct
    src = workloads.uniform_f32(6, M, D)
    oracle.scatter(table, idx, src)
    assert np.array_equal(oracle.gather(table, idx), src)
    untouched = np.ones(N, dtype=bool)
    untouched[idx] = False
    assert np.array_equal(table[untouched], before[untouched])


def test_two_byte_elements_and_bit_patterns():
    table = np.zeros((50, 9), dtype=np.uint16)
    src = np.arange(0x7bf0, 0x7bf0 + 3 * 9, dtype=np.uint16).reshape(3, 9)   # crosses inf / NaN patterns
    oracle.scatter(table, np.array([49, 0, 7], dtype=np.int32), src)
    assert table[49].tolist() == src[0].tolist() and table[0].tolist() == src[1].tolist()
    assert table[7].tolist() == src[2].tolist() and int(table.astype(np.int64).sum()) == int(src.astype(np.int64).sum())


@pytest.mark.parametrize("bad", [-1, 20, 2**31 - 1])
def test_bad_id_reports_first_position_and_writes_nothing(bad):
    table = workloads.uniform_f32(7, 20, 5)
    before = table.copy()
    idx = np.arange(10, dtype=np.int64)
    idx[6] = bad
    idx[8] = bad
    with pytest.raises(oracle.OracleIndexError) as e:
        oracle.scatter(table, idx, workloads.uniform_f32(8, 10, 5))
    assert e.value.pos == 6 and np.array_equal(table, before)


def test_empty_scatter_is_a_no_op():
    table = workloads.uniform_f32(9, 4, 4)
    before = table.copy()
    oracle.scatter(table, np.empty(0, dtype=np.int64), np.empty((0, 4), dtype=np.float32))
    assert np.array_equal(table, before)


@pytest.mark.parametrize("D,pitch", [(3, 8), (100, 128), (602, 608), (7, 7)])
def test_pitched_scatter_matches_numpy_and_leaves_the_padding_alone(D, pitch):
    N, M = 400, 250
    padded = workloads.uniform_f32(31, N, pitch)
    want = padded.copy()
    idx = np.random.default_rng(32).permutation(N)[:M].astype(np.int64)
    src = workloads.uniform_f32(33, M, D)
    oracle.scatter_raw(padded.ctypes.data, N, D, oracle.F32, idx, src, pitch=pitch)
    want[idx, :D] = src
    assert np.array_equal(padded.view(np.uint32), want.view(np.uint32))
