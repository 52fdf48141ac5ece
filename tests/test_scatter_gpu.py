"""GPU parity of the write direction (ud_scatter) against the oracle, bit for bit."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ud():
    import paper_2101_07956_amd as m
    return m


def distinct_ids(seed, M, N, dtype=np.int64):
    return np.random.default_rng(seed).permutation(N)[:M].astype(dtype)


def run_scatter(ud, table, idx_np, src_np, tuning=None):
    dtype = ud.UD_F32 if src_np.dtype.itemsize == 4 else ud.UD_F16
    idx = torch.from_numpy(idx_np).cuda()
    src = torch.from_numpy(src_np.view(np.int32 if src_np.dtype.itemsize == 4 else np.int16)).cuda()
    s = torch.cuda.current_stream().cuda_stream
    ud.ud_scatter(table.device_ptr, table.N, table.D, dtype, idx.data_ptr(),
                  ud.UD_I64 if idx_np.dtype == np.int64 else ud.UD_I32, idx_np.size, src.data_ptr(), s, tuning)
    ud.ud_gather_status(s)


def bits(a):
    return a.view(np.uint32 if a.dtype.itemsize == 4 else np.uint16)


@pytest.mark.parametrize("D", [1, 3, 4, 5, 16, 64, 100, 127, 128, 129, 256, 513, 602, 603, 1031, 4099])
def test_f32_scatter_into_host_table(ud, D):
    N, M = 3001, 1777
    t = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(t.host_ptr, 500 + D, N * D)
    want = t.numpy().copy()
    for idt in (np.int64, np.int32):
        idx = distinct_ids(D, M, N, idt)
        if 0 not in idx and N - 1 not in idx:
            idx[:2] = [0, N - 1]                       # first and last table row: head/tail chunks at the table's ends
        src = workloads.uniform_f32(600 + D, M, D)
        run_scatter(ud, t, idx, src)
        oracle.scatter(want, idx, src)
        assert np.array_equal(bits(t.numpy()), bits(want)), (D, idt)
    t.free()


@pytest.mark.parametrize("D", [1, 3, 8, 9, 301, 602, 603])
def test_f16_scatter_into_host_table(ud, D):
    N, M = 2503, 1200
    t = ud.Table(N, D, ud.UD_F16)
    workloads.fill_normal_f16(t.host_ptr, 700 + D, N * D)
    want = t.numpy().copy()
    idx = distinct_ids(D, M, N, np.int32)
    src = workloads.normal_f16(800 + D, M, D)
    run_scatter(ud, t, idx, src)
    oracle.scatter(want, idx, src)
    assert np.array_equal(bits(t.numpy()), bits(want)), D
    t.free()


PLANS = [(1, 1), (2, 1), (4, 1), (1, 2), (2, 2), (1, 3), (1, 4)]


@pytest.mark.parametrize("u,p", PLANS)
def test_every_scatter_instantiation_and_group_size(ud, u, p):
    N, M = 1201, 900
    for elem, D in ((ud.UD_F32, 77), (ud.UD_F16, 75)):
        t = ud.Table(N, D, elem)
        for lanes in (1, 4, 16, 64):
            fill = workloads.uniform_f32 if elem == ud.UD_F32 else workloads.normal_f16
            t.numpy()[:] = fill(1, N, D)
            want = t.numpy().copy()
            idx = distinct_ids(lanes + u * 10 + p, M, N)
            src = fill(2 + lanes, M, D)
            run_scatter(ud, t, idx, src, ud.ud_tuning(lanes, p, u, 0, 0))
            oracle.scatter(want, idx, src)
            assert np.array_equal(bits(t.numpy()), bits(want)), (elem, lanes, u, p)
        t.free()


def test_scatter_into_hbm_table_then_gather_back(ud):
    N, D, M = 20_000, 100, 7001
    host = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(host.host_ptr, 9, N * D)
    dev = host.to_device()
    idx = distinct_ids(10, M, N)
    src = workloads.uniform_f32(11, M, D)
    run_scatter(ud, dev, idx, src)
    want = host.numpy().copy()
    oracle.scatter(want, idx, src)
    # read the whole HBM table back with the gather
    allrows = torch.arange(N, dtype=torch.int64, device="cuda")
    out = torch.empty((N, D), dtype=torch.float32, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    ud.ud_gather(dev.device_ptr, N, D, ud.UD_F32, allrows.data_ptr(), ud.UD_I64, N, out.data_ptr(), s)
    ud.ud_gather_status(s)
    assert np.array_equal(bits(out.cpu().numpy()), bits(want))
    dev.free()
    host.free()


def test_duplicate_ids_leave_one_of_the_candidates_per_element(ud):
    N, D, M = 50, 100, 400                                       # every row is hit about 8 times
    t = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(t.host_ptr, 12, N * D)
    before = t.numpy().copy()
    idx = workloads.indices_uniform(13, M, N)
    src = workloads.uniform_f32(14, M, D)
    run_scatter(ud, t, idx, src)
    after = t.numpy()
    for r in range(N):
        cand = src[idx == r]
        if cand.shape[0] == 0:
            assert np.array_equal(after[r], before[r])
        else:
            assert (after[r][None, :] == cand).any(axis=0).all(), r
    t.free()


def test_bad_ids_are_skipped_and_reported(ud):
    N, D, M = 300, 64, 200
    t = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(t.host_ptr, 15, N * D)
    want = t.numpy().copy()
    idx = distinct_ids(16, M, N)
    src = workloads.uniform_f32(17, M, D)
    bad = idx.copy()
    bad[[150, 20]] = [N, -1]
    with pytest.raises(ud.UdIndexError) as e:
        run_scatter(ud, t, bad, src)
    assert e.value.pos == 20
    good = np.ones(M, dtype=bool)
    good[[150, 20]] = False
    oracle.scatter(want, np.ascontiguousarray(idx[good]), np.ascontiguousarray(src[good]))
    assert np.array_equal(bits(t.numpy()), bits(want))       # rows with valid IDs written, nothing else touched
    t.free()


def test_empty_scatter(ud):
    t = ud.Table(8, 8, ud.UD_F32)
    workloads.fill_uniform_f32(t.host_ptr, 18, 64)
    before = t.numpy().copy()
    ud.ud_scatter(t.device_ptr, 8, 8, ud.UD_F32, None, ud.UD_I64, 0, None, None)
    ud.ud_gather_status(None)
    assert np.array_equal(t.numpy(), before)
    t.free()


@pytest.mark.parametrize("elem_name,D", [("UD_F32", 100), ("UD_F32", 602), ("UD_F16", 301)])
def test_scatter_into_padded_table(ud, elem_name, D):
    import ctypes
    elem = getattr(ud, elem_name)
    N, M = 3001, 1500
    t = ud.Table(N, D, elem, ud.UD_TABLE_PAD_ROWS)
    storage = np.frombuffer((ctypes.c_char * t.nbytes).from_address(t.host_ptr),
                            dtype=np.uint32 if elem == ud.UD_F32 else np.uint16).reshape(N, t.pitch)
    storage[:] = np.random.default_rng(D).integers(0, 60000, size=storage.shape).astype(storage.dtype)
    want = storage.copy()
    idx = distinct_ids(D, M, N)
    src = (workloads.uniform_f32(5, M, D) if elem == ud.UD_F32 else workloads.normal_f16(5, M, D))
    oracle.scatter_raw(want.ctypes.data, N, D, oracle.F32 if elem == ud.UD_F32 else oracle.F16, idx,
                       np.ascontiguousarray(src), pitch=t.pitch)
    dsrc = torch.from_numpy(src.view(np.int32 if elem == ud.UD_F32 else np.int16)).cuda()
    didx = torch.from_numpy(idx).cuda()
    s = torch.cuda.current_stream().cuda_stream
    ud.ud_scatter_pitched(t.device_ptr, N, D, t.pitch, elem, didx.data_ptr(), ud.UD_I64, M, dsrc.data_ptr(), s)
    ud.ud_gather_status(s)
    assert np.array_equal(storage, want)                      # data rows updated, padding and other rows untouched
    t.free()


@pytest.mark.parametrize("esz,D", [(2, 1), (2, 3), (2, 5), (2, 7), (4, 1), (4, 2), (4, 3)])
def test_rows_shorter_than_a_chunk_with_an_unaligned_table_base(ud, esz, D):
    # rows of 2..14 bytes: a 16-byte destination chunk then spans several table rows, and the source
    # elements beside a row's own may lie before the first or after the last source row; the source
    # buffer is placed at the very start and the very end of its allocation so that an over-read shows
    dtype = ud.UD_F32 if esz == 4 else ud.UD_F16
    npdt = np.uint32 if esz == 4 else np.uint16
    rng = np.random.default_rng(100 * esz + D)
    s = torch.cuda.current_stream().cuda_stream
    for shift in range(0, 16 // esz):
        for M in (1, 2, 3, 17, 298):
            N = 415
            big = ud.Table(N + 8, D, dtype)
            storage = np.frombuffer((__import__("ctypes").c_char * big.nbytes).from_address(big.host_ptr), dtype=npdt)
            storage[:] = rng.integers(0, 2 ** (8 * esz), size=storage.size, dtype=np.uint64).astype(npdt)
            want_all = storage.copy()
            idx = rng.permutation(N)[:M].astype(np.int64)
            end_row = 0 if shift % 2 else N - 1               # the first or the last table row, IDs kept distinct
            if end_row in idx:
                idx[idx == end_row] = idx[0]
            idx[0] = end_row
            src = rng.integers(0, 2 ** (8 * esz), size=(M, D), dtype=np.uint64).astype(npdt)
            oracle.scatter(want_all[shift:shift + N * D].reshape(N, D), idx, src)
            dsrc = torch.from_numpy(src.view(np.int32 if esz == 4 else np.int16)).cuda()
            didx = torch.from_numpy(idx).cuda()
            before = storage.copy()
            for tun in (None, ud.ud_tuning(0, 1, 0, 0, ud.UD_TUNE_FLAT_SOURCE), ud.ud_tuning(0, 4, 0, 0, ud.UD_TUNE_FLAT_SOURCE)):
                storage[:] = before
                ud.ud_scatter(big.device_ptr + shift * esz, N, D, dtype, didx.data_ptr(), ud.UD_I64, M, dsrc.data_ptr(), s, tun)
                ud.ud_gather_status(s)
                assert np.array_equal(storage, want_all), (esz, D, shift, M, tun and tun.flags)
            big.free()


# ---- the source-aligned kernel (automatic for tables in HBM; UD_TUNE_FLAT_SOURCE elsewhere) ----

@pytest.mark.parametrize("P", [1, 2, 4])
def test_source_aligned_scatter_every_instantiation(ud, P):
    # fp32 and fp16, int64 and int32 IDs, widths below / at / above a wavefront tile and rows shorter than a chunk,
    # host and HBM tables, source buffers at every alignment of the 16-byte chunk grid, capped grid
    N, M = 1201, 1103
    s = torch.cuda.current_stream().cuda_stream
    for elem, D in ((ud.UD_F32, 77), (ud.UD_F32, 2), (ud.UD_F32, 1030), (ud.UD_F32, 100), (ud.UD_F16, 75), (ud.UD_F16, 7),
                    (ud.UD_F16, 2051), (ud.UD_F16, 301)):
        esz = 4 if elem == ud.UD_F32 else 2
        fill = workloads.uniform_f32 if elem == ud.UD_F32 else workloads.normal_f16
        host = ud.Table(N, D, elem)
        host.numpy()[:] = fill(1, N, D)
        dev = host.to_device()
        for idt in (np.int64, np.int32):
            idx = distinct_ids(D + P, M, N, idt)
            idx[:2] = [0, N - 1] if 0 not in idx[2:] and N - 1 not in idx[2:] else idx[:2]
            src = fill(3 + P, M, D)
            want = host.numpy().copy()
            oracle.scatter(want, idx, src)
            didx = torch.from_numpy(idx).cuda()
            for off in (0, 1, 16 // esz - 1):
                buf = torch.zeros(M * D + 16, dtype=torch.int32 if esz == 4 else torch.int16, device="cuda")
                buf[off:off + M * D] = torch.from_numpy(src.view(np.int32 if esz == 4 else np.int16).ravel()).cuda()
                for blocks, nt in ((0, 0), (3, ud.UD_TUNE_NT_STORE)):
                    tun = ud.ud_tuning(0, P, 0, blocks, ud.UD_TUNE_FLAT_SOURCE | nt)
                    # host table through the flag
                    host.numpy()[:] = fill(1, N, D)
                    ud.ud_scatter(host.device_ptr, N, D, elem, didx.data_ptr(), ud.UD_I64 if idt == np.int64 else ud.UD_I32, M,
                                  buf.data_ptr() + off * esz, s, tun)
                    ud.ud_gather_status(s)
                    assert np.array_equal(bits(host.numpy()), bits(want)), (elem, D, idt, off, blocks)
            # HBM table: the automatic choice; read back with the gather
            ud.ud_scatter(dev.device_ptr, N, D, elem, didx.data_ptr(), ud.UD_I64 if idt == np.int64 else ud.UD_I32, M,
                          torch.from_numpy(src.view(np.int32 if esz == 4 else np.int16)).cuda().data_ptr(), s)
            allrows = torch.arange(N, dtype=torch.int64, device="cuda")
            out = torch.empty((N, D), dtype=torch.float32 if esz == 4 else torch.float16, device="cuda")
            ud.ud_gather(dev.device_ptr, N, D, elem, allrows.data_ptr(), ud.UD_I64, N, out.data_ptr(), s)
            ud.ud_gather_status(s)
            assert np.array_equal(bits(out.cpu().numpy()), bits(want)), (elem, D, idt, "hbm")
            # put the HBM copy back for the next ID type
            host.numpy()[:] = fill(1, N, D)
            dev.free()
            dev = host.to_device()
        dev.free()
        host.free()


def test_source_aligned_scatter_skips_and_reports_bad_ids(ud):
    N, D, M = 300, 602, 200
    t = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(t.host_ptr, 15, N * D)
    want = t.numpy().copy()
    idx = distinct_ids(16, M, N)
    src = workloads.uniform_f32(17, M, D)
    bad = idx.copy()
    bad[[150, 20]] = [N, -1]
    with pytest.raises(ud.UdIndexError) as e:
        run_scatter(ud, t, bad, src, ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_FLAT_SOURCE))
    assert e.value.pos == 20
    good = np.ones(M, dtype=bool)
    good[[150, 20]] = False
    oracle.scatter(want, idx[good], src[good])
    assert np.array_equal(bits(t.numpy()), bits(want))          # rows of bad IDs untouched, every other row written
    t.free()


def test_very_wide_rows_are_scattered_whole(ud):
    # 400 KB rows: many chunk blocks per row in the row-per-lane-group kernel, a row far longer than a wavefront
    # tile in the source-aligned one; host table, then its HBM copy read back through the gather
    N, D, M = 37, 100_003, 29
    t = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(t.host_ptr, 90, N * D)
    dev = t.to_device()
    idx = distinct_ids(91, M, N)
    src = workloads.uniform_f32(92, M, D)
    want = t.numpy().copy()
    oracle.scatter(want, idx, src)
    run_scatter(ud, t, idx, src)
    assert np.array_equal(bits(t.numpy()), bits(want))
    for tun in (None, ud.ud_tuning(0, 4, 0, 7, ud.UD_TUNE_FLAT_SOURCE)):
        run_scatter(ud, dev, idx, src, tun)
        allrows = torch.arange(N, dtype=torch.int64, device="cuda")
        out = torch.empty((N, D), dtype=torch.float32, device="cuda")
        s = torch.cuda.current_stream().cuda_stream
        ud.ud_gather(dev.device_ptr, N, D, ud.UD_F32, allrows.data_ptr(), ud.UD_I64, N, out.data_ptr(), s)
        ud.ud_gather_status(s)
        assert np.array_equal(bits(out.cpu().numpy()), bits(want))
    dev.free()
    t.free()


def test_full_size_scatter_into_the_benchmark_table(ud):
    # the write direction at the benchmark's size: 1,000,000 distinct rows x 602 fp32 into the 4,000,000-row
    # host-pinned table (9.6 GB), the whole table compared with the oracle's; then the same into its HBM copy,
    # read back through the gather
    N, D, M = 4_000_000, 602, 1_000_000
    t = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(t.host_ptr, 8, N * D)
    dev = t.to_device()
    idx = np.random.default_rng(8).permutation(N)[:M].astype(np.int64)
    if 0 not in idx:
        idx[0] = 0                                              # the table's first and last rows take part
    if N - 1 not in idx:
        idx[1] = N - 1
    src = workloads.uniform_f32(81, M, D)
    dsrc, didx = torch.from_numpy(src).cuda(), torch.from_numpy(idx).cuda()
    s = torch.cuda.current_stream().cuda_stream
    want = t.numpy().copy()                                     # 9.6 GB on the host
    oracle.scatter(want, idx, src)
    print("full-size scatter: oracle done", flush=True)
    ud.ud_scatter(t.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, dsrc.data_ptr(), s)
    ud.ud_gather_status(s)
    assert np.array_equal(bits(t.numpy()), bits(want))
    del want
    # HBM copy: scatter, then compare the written rows and a sample of untouched rows through the gather
    ud.ud_scatter(dev.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, dsrc.data_ptr(), s)
    out = torch.empty((M, D), dtype=torch.float32, device="cuda")
    ud.ud_gather(dev.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, out.data_ptr(), s)
    ud.ud_gather_status(s)
    assert torch.equal(out, dsrc)
    others = np.setdiff1d(np.random.default_rng(9).integers(0, N, 300_000), idx)[:100_000].astype(np.int64)
    dothers = torch.from_numpy(others).cuda()
    ud.ud_gather(dev.device_ptr, N, D, ud.UD_F32, dothers.data_ptr(), ud.UD_I64, others.size, out.data_ptr(), s)
    ud.ud_gather_status(s)
    assert np.array_equal(bits(out[: others.size].cpu().numpy()), bits(t.numpy()[others]))   # t now equals the oracle's table
    dev.free()
    t.free()
