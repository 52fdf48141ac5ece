"""GPU parity: the HIP gather, called through the C ABI, against the CPU oracle.

Bit-exact comparison (integer/bit work: the gather copies patterns, the
widening is exact), on seeded inputs that span several wavefront batches and a
ragged tail, for every kernel instantiation the library can select.
"""
import ctypes
import itertools

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


CANARY = 0x5A


def run_gather(ud, table, idx_np, dtype, tuning=None, out_offset_elems=0):
    """Gather on the GPU into a canary-filled buffer; returns the (M, D) result as raw bits."""
    M = idx_np.size
    obytes = 2 if dtype == ud.UD_F16 else 4
    pad = 64
    total = M * table.D + out_offset_elems + pad
    buf = torch.full((total * obytes,), CANARY, dtype=torch.uint8, device="cuda")
    idx = torch.from_numpy(idx_np).cuda()
    out_ptr = buf.data_ptr() + out_offset_elems * obytes
    stream = torch.cuda.current_stream().cuda_stream
    ud.ud_gather_tuned(table.device_ptr, table.N, table.D, dtype, idx.data_ptr(),
                       ud.UD_I64 if idx_np.dtype == np.int64 else ud.UD_I32, M, out_ptr, stream, tuning)
    ud.ud_gather_status(stream)
    host = buf.cpu().numpy()
    lo = out_offset_elems * obytes
    hi = lo + M * table.D * obytes
    assert (host[:lo] == CANARY).all(), "wrote before the output"
    assert (host[hi:] == CANARY).all(), "wrote past the output"
    return host[lo:hi].view(np.uint16 if obytes == 2 else np.uint32).reshape(M, table.D)


def oracle_bits(table_np, idx_np, dtype):
    o = oracle.gather(table_np, idx_np, dtype)
    return o.view(np.uint16 if o.dtype.itemsize == 2 else np.uint32)


def make_table(ud, N, D, elem, seed, flags=0):
    t = ud.Table(N, D, elem, flags)
    if elem == ud.UD_F32:
        workloads.fill_uniform_f32(t.host_ptr, seed, N * D)
    else:
        workloads.fill_normal_f16(t.host_ptr, seed, N * D)
    return t


def test_config1_single_gather(ud):
    # fp32 100,000 x 128, uniform[-1,1) seed 0; 16,384 int64 IDs uniform with replacement
    t = make_table(ud, 100_000, 128, ud.UD_F32, 0)
    idx = workloads.indices_uniform(workloads.IDX_STREAM, 16_384, 100_000)
    got = run_gather(ud, t, idx, ud.UD_F32)
    assert np.array_equal(got, oracle_bits(t.numpy(), idx, oracle.F32))
    t.free()


WIDTHS = [1, 2, 3, 4, 5, 7, 16, 25, 64, 100, 127, 128, 129, 255, 256, 257, 300, 512, 513, 514, 515, 516, 517, 518, 519,
          602, 603, 1031, 4096, 4099]          # 512..519 are the row sizes 2048..2076 bytes of the paper's Figure 7


@pytest.mark.parametrize("D", WIDTHS)
def test_f32_widths_default_plan(ud, D):
    N, M = 3001, 2377                      # M is no multiple of any rows-per-wavefront
    t = make_table(ud, N, D, ud.UD_F32, 100 + D)
    for idt in (np.int64, np.int32):
        idx = workloads.indices_uniform(7, M, N, idt)
        idx[:3] = [0, N - 1, N - 1]        # first and last row, head and tail chunks at the table's ends
        got = run_gather(ud, t, idx, ud.UD_F32, out_offset_elems=D % 4)
        assert np.array_equal(got, oracle_bits(t.numpy(), idx, oracle.F32)), (D, idt)
    t.free()


@pytest.mark.parametrize("D", [1, 3, 8, 9, 100, 301, 602, 603, 1027])
@pytest.mark.parametrize("dtype_name", ["UD_F16", "UD_F16_TO_F32"])
def test_f16_widths_default_plan(ud, D, dtype_name):
    dtype = getattr(ud, dtype_name)
    N, M = 2503, 1999
    t = make_table(ud, N, D, ud.UD_F16, 200 + D)
    idx = workloads.indices_uniform(8, M, N, np.int32)
    idx[:3] = [0, N - 1, N - 1]
    got = run_gather(ud, t, idx, dtype, out_offset_elems=D % 3)
    assert np.array_equal(got, oracle_bits(t.numpy(), idx, dtype)), D
    t.free()


PLANS = [(u, p) for u, p in itertools.product((1, 2, 4), (1, 2, 3, 4)) if u * p <= 8 and (u, p) != (4, 2)]


@pytest.mark.parametrize("u,p", PLANS)
def test_every_instantiation_every_group_size(ud, u, p):
    # each (rows in flight, chunks per lane) kernel with each lane-group size, with and
    # without streaming stores, on a width whose rows start at 4 different offsets mod 16
    N, M = 1201, 1103
    cases = [(ud.UD_F32, ud.UD_F32, 77), (ud.UD_F16, ud.UD_F16_TO_F32, 301), (ud.UD_F16, ud.UD_F16, 75)]
    for elem, dtype, D in cases:
        t = make_table(ud, N, D, elem, 300 + D)
        idx = workloads.indices_uniform(9, M, N)
        want = oracle_bits(t.numpy(), idx, dtype)
        for lanes in (1, 2, 4, 8, 16, 32, 64):
            for flags in (0, ud.UD_TUNE_NT_STORE):
                tun = ud.ud_tuning(lanes, p, u, 0, flags)
                got = run_gather(ud, t, idx, dtype, tun)
                assert np.array_equal(got, want), (dtype, D, lanes, u, p, flags)
        t.free()


def test_grid_stride_when_blocks_are_capped(ud):
    N, D, M = 5000, 100, 40_000
    t = make_table(ud, N, D, ud.UD_F32, 5)
    idx = workloads.indices_uniform(10, M, N)
    want = oracle_bits(t.numpy(), idx, oracle.F32)
    for blocks in (1, 7, 256):
        for flags in (0, ud.UD_TUNE_DEST_ALIGNED, ud.UD_TUNE_DEST_ALIGNED | ud.UD_TUNE_NT_STORE):
            got = run_gather(ud, t, idx, ud.UD_F32, ud.ud_tuning(0, 0, 0, blocks, flags))
            assert np.array_equal(got, want), (blocks, flags)
    t.free()


@pytest.mark.parametrize("dtype_name,elem_name,D", [("UD_F32", "UD_F32", 37), ("UD_F16_TO_F32", "UD_F16", 301),
                                                     ("UD_F16", "UD_F16", 33)])
def test_elementwise_kernel(ud, dtype_name, elem_name, D):
    dtype, elem = getattr(ud, dtype_name), getattr(ud, elem_name)
    N, M = 777, 1500
    t = make_table(ud, N, D, elem, 6)
    idx = workloads.indices_uniform(11, M, N, np.int32)
    want = oracle_bits(t.numpy(), idx, dtype)
    got = run_gather(ud, t, idx, dtype, ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_ELEMENTWISE))
    assert np.array_equal(got, want)
    # the paper's circular shift changes which lane moves which element, never the result
    got = run_gather(ud, t, idx, dtype, ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_ELEMENTWISE | ud.UD_TUNE_CIRCULAR_SHIFT))
    assert np.array_equal(got, want)
    t.free()


@pytest.mark.parametrize("D", [1, 3, 11, 63, 64, 65, 100, 512, 513, 514, 515, 516, 517, 518, 519, 602])
def test_one_lane_per_element_and_circular_shift_kernel_widths(ud, D):
    # the paper's two thread layouts (Figures 4 and 5), among others on all eight row sizes of its Figure 7
    N, M = 1501, 2203
    t = make_table(ud, N, D, ud.UD_F32, 700 + D)
    idx = workloads.indices_uniform(12, M, N)
    want = oracle_bits(t.numpy(), idx, oracle.F32)
    for flags in (ud.UD_TUNE_ELEMENTWISE, ud.UD_TUNE_ELEMENTWISE | ud.UD_TUNE_CIRCULAR_SHIFT):
        assert np.array_equal(run_gather(ud, t, idx, ud.UD_F32, ud.ud_tuning(0, 0, 0, 0, flags)), want), (D, flags)
    t.free()


@pytest.mark.parametrize("D", [16, 64, 100, 256, 602])
def test_share_gpu_launch_shape(ud, D):
    N, M = 20_000, 30_011
    t = make_table(ud, N, D, ud.UD_F32, 30 + D)
    idx = workloads.indices_uniform(31, M, N)
    got = run_gather(ud, t, idx, ud.UD_F32, ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_SHARE_GPU))
    assert np.array_equal(got, oracle_bits(t.numpy(), idx, oracle.F32)), D
    t.free()


def test_index_patterns(ud):
    N, D = 4099, 100
    t = make_table(ud, N, D, ud.UD_F32, 12)
    tab = t.numpy()
    got = run_gather(ud, t, np.arange(N, dtype=np.int64), ud.UD_F32)
    assert got.tobytes() == tab.tobytes()                       # arange is the identity
    got = run_gather(ud, t, np.full(3000, 1234, dtype=np.int64), ud.UD_F32)
    assert (got == tab[1234].view(np.uint32)).all()             # all-equal IDs
    got = run_gather(ud, t, np.full(777, N - 1, dtype=np.int32), ud.UD_F32)
    assert (got == tab[N - 1].view(np.uint32)).all()            # last row only
    idx = workloads.indices_uniform(13, 5000, N)
    perm = np.random.default_rng(0).permutation(idx.size)
    a = run_gather(ud, t, idx, ud.UD_F32)
    b = run_gather(ud, t, idx[perm], ud.UD_F32)
    assert np.array_equal(a[perm], b)                           # permuting IDs permutes rows
    t.free()


def test_tag_table_closed_form(ud):
    N, D = 70_001, 602
    t = ud.Table(N, D, ud.UD_F32)
    workloads.fill_tag(t.host_ptr, N * D, 4)
    idx = workloads.indices_uniform(14, 30_011, N)
    got = run_gather(ud, t, idx, ud.UD_F32).astype(np.int64)
    assert np.array_equal(got, idx[:, None] * D + np.arange(D)[None, :])
    t.free()


def test_all_65536_half_patterns_widen_exactly(ud):
    t = ud.Table(256, 256, ud.UD_F16)
    t.numpy().view(np.uint16)[:] = np.arange(65536, dtype=np.uint32).astype(np.uint16).reshape(256, 256)
    for idx in (np.arange(256, dtype=np.int64), np.random.default_rng(1).permutation(256).astype(np.int64)):
        want = oracle_bits(t.numpy(), idx, oracle.F16_TO_F32)
        assert np.array_equal(run_gather(ud, t, idx, ud.UD_F16_TO_F32), want)
        assert np.array_equal(run_gather(ud, t, idx, ud.UD_F16_TO_F32, ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_ELEMENTWISE)), want)
        assert np.array_equal(run_gather(ud, t, idx, ud.UD_F16), t.numpy().view(np.uint16)[idx])
    t.free()


def test_special_fp32_patterns_pass_unchanged(ud):
    pats = np.array([0x7fc00001, 0xffc12345, 0x7f800001, 0x80000000, 0x00000001, 0x7f800000, 0xff800000, 0x807fffff,
                     0x00000000, 0xffffffff], dtype=np.uint32)
    t = ud.Table(64, 10, ud.UD_F32)
    t.numpy().view(np.uint32)[:] = np.stack([np.roll(pats, k) for k in range(64)])
    idx = workloads.indices_uniform(15, 500, 64)
    assert np.array_equal(run_gather(ud, t, idx, ud.UD_F32), t.numpy().view(np.uint32)[idx])
    t.free()


@pytest.mark.parametrize("shift_elems", [1, 2, 3])
def test_table_base_not_16_byte_aligned(ud, shift_elems):
    # a raw table pointer that is only element-aligned: rows of a larger allocation, offset by a few elements
    N, D = 1000, 37
    big = ud.Table(N + 1, D, ud.UD_F32)
    workloads.fill_uniform_f32(big.host_ptr, 16, (N + 1) * D)
    flat = big.numpy().ravel()
    view = flat[shift_elems:shift_elems + N * D].reshape(N, D)
    idx = workloads.indices_uniform(17, 1500, N)
    idx[:2] = [0, N - 1]
    M = idx.size
    out = torch.full((M * D + 16,), -1, dtype=torch.int32, device="cuda")
    didx = torch.from_numpy(idx).cuda()
    s = torch.cuda.current_stream().cuda_stream
    ud.ud_gather(big.device_ptr + 4 * shift_elems, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, out.data_ptr(), s)
    ud.ud_gather_status(s)
    host = out.cpu().numpy()
    assert (host[M * D:] == -1).all()
    assert np.array_equal(host[:M * D].view(np.uint32).reshape(M, D), oracle_bits(np.ascontiguousarray(view), idx, oracle.F32))
    big.free()


def test_noncoherent_host_table_and_device_resident_table(ud):
    N, D, M = 20_000, 256, 9001
    for flags in (ud.UD_TABLE_COHERENT, ud.UD_TABLE_NONCOHERENT):
        t = make_table(ud, N, D, ud.UD_F32, 18, flags)
        idx = workloads.indices_uniform(19, M, N)
        want = oracle_bits(t.numpy(), idx, oracle.F32)
        assert np.array_equal(run_gather(ud, t, idx, ud.UD_F32), want)
        dev = t.to_device()
        assert dev.host_ptr == 0 and dev.N == N and dev.D == D
        assert np.array_equal(run_gather(ud, dev, idx, ud.UD_F32), want)
        # a slice of rows held in HBM: IDs are relative to the slice
        part = t.to_device(5000, 4000)
        idx2 = workloads.indices_uniform(20, 3000, 4000)
        assert np.array_equal(run_gather(ud, part, idx2, ud.UD_F32), oracle_bits(t.numpy()[5000:9000], idx2, oracle.F32))
        for x in (part, dev, t):
            x.free()


def test_empty_id_list_is_a_no_op(ud):
    t = make_table(ud, 10, 8, ud.UD_F32, 21)
    out = torch.full((8,), 7, dtype=torch.int32, device="cuda")
    ud.ud_gather(t.device_ptr, 10, 8, ud.UD_F32, None, ud.UD_I64, 0, out.data_ptr(), None)
    ud.ud_gather_status(None)
    assert (out.cpu().numpy() == 7).all()
    t.free()


@pytest.mark.parametrize("idt", [np.int64, np.int32])
@pytest.mark.parametrize("elementwise", [False, True])
def test_out_of_range_ids_are_reported_and_never_dereferenced(ud, idt, elementwise):
    N, D, M = 500, 100, 4000
    t = make_table(ud, N, D, ud.UD_F32, 22)
    tun = ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_ELEMENTWISE if elementwise else 0)
    idx = workloads.indices_uniform(23, M, N, idt)
    for bad_positions, bad_values in (([3111, 1717, 2500], [N, -1, N + 5]), ([0], [-7]), ([M - 1], [2**31 - 1])):
        bad = idx.copy()
        bad[bad_positions] = bad_values
        with pytest.raises(ud.UdIndexError) as e:
            run_gather(ud, t, bad, ud.UD_F32, tun)
        assert e.value.pos == min(bad_positions)
        with pytest.raises(oracle.OracleIndexError) as oe:          # the oracle reports the same position
            oracle.gather(t.numpy(), bad)
        assert oe.value.pos == e.value.pos
        # the record is cleared by the status call: a clean gather afterwards passes
        assert np.array_equal(run_gather(ud, t, idx, ud.UD_F32, tun), oracle_bits(t.numpy(), idx, oracle.F32))
    if idt == np.int64:
        bad = idx.copy()
        bad[10] = 2**32 + 3                                          # would alias row 3 if truncated to 32 bits
        with pytest.raises(ud.UdIndexError) as e:
            run_gather(ud, t, bad, ud.UD_F32, tun)
        assert e.value.pos == 10
    t.free()


def test_rows_with_valid_ids_are_still_gathered_when_another_id_is_bad(ud):
    N, D, M = 300, 64, 1000
    t = make_table(ud, N, D, ud.UD_F32, 24)
    idx = workloads.indices_uniform(25, M, N)
    idx[500] = N
    out = torch.zeros((M, D), dtype=torch.float32, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, torch.from_numpy(idx).cuda().data_ptr(), ud.UD_I64, M, out.data_ptr(), s)
    with pytest.raises(ud.UdIndexError):
        ud.ud_gather_status(s)
    host = out.cpu().numpy()
    good = np.ones(M, dtype=bool)
    good[500] = False
    assert np.array_equal(host[good], t.numpy()[idx[good]])
    assert (host[500] == 0).all()                                    # the bad row is left unwritten
    t.free()


def test_plan_depends_on_where_the_table_lives(ud):
    t = make_table(ud, 5000, 128, ud.UD_F32, 26)
    host_plan = ud.ud_gather_plan(t.device_ptr, 128, ud.UD_F32)
    assert host_plan.lanes_per_row == 64 and host_plan.rows_in_flight == 1 and host_plan.flags == 0
    d = t.to_device()
    dev_plan = ud.ud_gather_plan(d.device_ptr, 128, ud.UD_F32)
    assert dev_plan.flags & ud.UD_TUNE_DEST_ALIGNED and dev_plan.chunks_per_lane in (1, 2, 4)
    # a pointer into the middle of a table the library made is recognised too
    mid_plan = ud.ud_gather_plan(d.device_ptr + 128 * 4 * 100, 128, ud.UD_F32)
    assert mid_plan.flags == dev_plan.flags
    # explicit tuning without the flag selects the source-aligned kernel on the same table
    idx = workloads.indices_uniform(27, 3000, 5000)
    want = oracle_bits(t.numpy(), idx, oracle.F32)
    for tun in (ud.ud_tuning(0, 0, 0, 0, 0), ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_NT_STORE),
                ud.ud_tuning(0, 0, 0, 0, dev_plan.flags), None):
        assert np.array_equal(run_gather(ud, d, idx, ud.UD_F32, tun), want)
    d.free()
    t.free()


# ---- hot-row cache (hybrid placement): same results as the plain gather ----

def run_cached(ud, cache, dtype, idx_np, D):
    M = idx_np.size
    obytes = 2 if dtype == ud.UD_F16 else 4
    buf = torch.full(((M * D + 64) * obytes,), CANARY, dtype=torch.uint8, device="cuda")
    idx = torch.from_numpy(idx_np).cuda()
    s = torch.cuda.current_stream().cuda_stream
    ud.ud_gather_cached(cache.handle, dtype, idx.data_ptr(), ud.UD_I64 if idx_np.dtype == np.int64 else ud.UD_I32,
                        M, buf.data_ptr(), s)
    ud.ud_gather_status(s)
    host = buf.cpu().numpy()
    assert (host[M * D * obytes:] == CANARY).all()
    return host[: M * D * obytes].view(np.uint16 if obytes == 2 else np.uint32).reshape(M, D)


@pytest.mark.parametrize("D", [16, 100, 128, 602])
def test_cached_gather_equals_oracle_fp32(ud, D):
    N, M = 30_011, 20_003
    t = make_table(ud, N, D, ud.UD_F32, 400 + D)
    rng = np.random.default_rng(D)
    for n_hot in (1, 977, N):                                   # one row, a few, every row
        hot = rng.permutation(N)[:n_hot].astype(np.int64)
        c = ud.Cache(t, hot)
        for idt in (np.int64, np.int32):
            idx = workloads.indices_uniform(40 + n_hot, M, N, idt)
            idx[: min(n_hot, 50)] = hot[: min(n_hot, 50)]       # make sure cached rows are hit
            idx[-2:] = [0, N - 1]
            got = run_cached(ud, c, ud.UD_F32, idx, D)
            assert np.array_equal(got, oracle_bits(t.numpy(), idx, oracle.F32)), (D, n_hot, idt)
        c.free()
    t.free()


def test_cached_gather_reads_the_cached_copy(ud):
    # after the cache is built the host rows are overwritten: cached rows must come from HBM
    # (old values), uncached rows over the link (new values)
    N, D, M = 5000, 64, 4000
    t = make_table(ud, N, D, ud.UD_F32, 41)
    old = t.numpy().copy()
    hot = np.arange(0, N, 3, dtype=np.int64)
    c = ud.Cache(t, hot)
    t.numpy()[:] = old + 1.0
    idx = workloads.indices_uniform(42, M, N)
    got = run_cached(ud, c, ud.UD_F32, idx, D).view(np.float32)
    is_hot = (idx % 3) == 0
    assert is_hot.any() and (~is_hot).any()
    assert np.array_equal(got[is_hot], old[idx[is_hot]])
    assert np.array_equal(got[~is_hot], (old + 1.0)[idx[~is_hot]])
    c.free()
    t.free()


def test_cached_gather_fp16_and_errors(ud):
    N, D, M = 9001, 301, 7000
    t = make_table(ud, N, D, ud.UD_F16, 43)
    hot = workloads.indices_uniform(44, 2000, N)                # duplicates tolerated
    c = ud.Cache(t, hot)
    idx = workloads.indices_uniform(45, M, N, np.int32)
    for dtype in (ud.UD_F16, ud.UD_F16_TO_F32):
        assert np.array_equal(run_cached(ud, c, dtype, idx, D), oracle_bits(t.numpy(), idx, dtype))
    bad = idx.copy()
    bad[1234] = N
    with pytest.raises(ud.UdIndexError) as e:
        run_cached(ud, c, ud.UD_F16, bad, D)
    assert e.value.pos == 1234
    with pytest.raises(ud.UdError):                             # fp32 gather on an fp16 table
        ud.ud_gather_cached(c.handle, ud.UD_F32, 0x1000, ud.UD_I64, 1, 0x2000, None)
    with pytest.raises(ud.UdError):                             # hot row out of range
        ud.Cache(t, np.array([0, N], dtype=np.int64))
    c.free()
    t.free()


def test_more_rows_than_the_workgroup_cap_and_offsets_beyond_32_bits(ud):
    # 17,000,000 rows of 256 bytes: one wavefront per row would need more workgroups than the
    # launch cap, so the kernel strides; output offsets pass 4 GiB
    N, D, M = 200_000, 64, 17_000_000
    t = make_table(ud, N, D, ud.UD_F32, 50)
    idx = workloads.indices_uniform(51, M, N)
    didx = torch.from_numpy(idx).cuda()
    out = torch.empty(M * D + 16, dtype=torch.int32, device="cuda")
    out[M * D:] = 0x5A5A5A5A
    s = torch.cuda.current_stream().cuda_stream
    ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, out.data_ptr(), s)
    ud.ud_gather_status(s)
    want = np.empty((M, D), dtype=np.uint32)
    oracle.gather_raw(t.host_ptr, N, D, oracle.F32, idx, want)
    host = out.cpu().numpy().view(np.uint32)
    assert (host[M * D:] == 0x5A5A5A5A).all()
    assert np.array_equal(host[: M * D].reshape(M, D), want)
    t.free()


def test_single_row_table_and_single_id(ud):
    t = make_table(ud, 1, 602, ud.UD_F32, 52)
    got = run_gather(ud, t, np.zeros(1, dtype=np.int64), ud.UD_F32)
    assert np.array_equal(got, t.numpy().view(np.uint32))
    got = run_gather(ud, t, np.zeros(333, dtype=np.int32), ud.UD_F32)
    assert (got == t.numpy().view(np.uint32)).all()
    t.free()


def test_very_wide_rows(ud):
    N, D, M = 37, 100_003, 29                  # 400 KB rows: many chunk blocks per row, a row far longer than a wavefront tile
    t = make_table(ud, N, D, ud.UD_F32, 53)
    idx = workloads.indices_uniform(54, M, N)
    want = oracle_bits(t.numpy(), idx, oracle.F32)
    assert np.array_equal(run_gather(ud, t, idx, ud.UD_F32), want)
    dev = t.to_device()                         # the destination-aligned kernel
    assert np.array_equal(run_gather(ud, dev, idx, ud.UD_F32), want)
    for P in (1, 4):
        assert np.array_equal(run_gather(ud, dev, idx, ud.UD_F32, tuning=ud.ud_tuning(0, P, 0, 5, ud.UD_TUNE_DEST_ALIGNED)), want)
    dev.free()
    t.free()
    # the same in half precision, widened: 200 KB rows in, 400 KB rows out
    t = make_table(ud, N, D, ud.UD_F16, 55)
    want = oracle_bits(t.numpy(), idx, oracle.F16_TO_F32)
    assert np.array_equal(run_gather(ud, t, idx, ud.UD_F16_TO_F32), want)
    dev = t.to_device()
    assert np.array_equal(run_gather(ud, dev, idx, ud.UD_F16_TO_F32), want)
    dev.free()
    t.free()


def test_id_list_may_live_in_pinned_host_memory(ud):
    # ud_gather needs device-dereferenceable pointers only: the ID list itself can stay in mapped host memory
    N, D, M = 10_000, 128, 6001
    t = make_table(ud, N, D, ud.UD_F32, 60)
    ids_mem = ud.Table(1, 2 * M, ud.UD_F32)                       # M int64 slots of mapped host memory
    idx = workloads.indices_uniform(61, M, N)
    ids_mem.numpy().view(np.int64)[0, :] = idx
    out = torch.empty((M, D), dtype=torch.float32, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, ids_mem.device_ptr, ud.UD_I64, M, out.data_ptr(), s)
    ud.ud_gather_status(s)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), oracle_bits(t.numpy(), idx, oracle.F32))
    ids_mem.free()
    t.free()


def test_two_streams_gather_concurrently(ud):
    N, D, M = 50_000, 256, 40_000
    t = make_table(ud, N, D, ud.UD_F32, 62)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    idxs = [workloads.indices_uniform(63 + k, M, N) for k in range(2)]
    didx = [torch.from_numpy(a).cuda() for a in idxs]
    outs = [torch.empty((M, D), dtype=torch.float32, device="cuda") for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(3):
        for k in range(2):
            ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, didx[k].data_ptr(), ud.UD_I64, M, outs[k].data_ptr(),
                         streams[k].cuda_stream)
    for k in range(2):
        ud.ud_gather_status(streams[k].cuda_stream)
        assert np.array_equal(outs[k].cpu().numpy().view(np.uint32), oracle_bits(t.numpy(), idxs[k], oracle.F32))
    t.free()


def test_id_errors_are_recorded_per_stream(ud):
    N, D, M = 20_000, 256, 200_000
    t = make_table(ud, N, D, ud.UD_F32, 66)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    good = workloads.indices_uniform(67, M, N)
    bad_a, bad_b = good.copy(), good.copy()
    bad_a[777] = -5
    bad_b[M - 3] = N
    d_good, d_a, d_b = (torch.from_numpy(x).cuda() for x in (good, bad_a, bad_b))
    outs = [torch.empty((M, D), dtype=torch.float32, device="cuda") for _ in range(2)]
    torch.cuda.synchronize()

    def launch(stream, ids, out):
        ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, ids.data_ptr(), ud.UD_I64, M, out.data_ptr(), stream.cuda_stream)

    # a bad ID on stream A only: B reports nothing, A reports its position, then A is clean again
    launch(sa, d_a, outs[0])
    launch(sb, d_good, outs[1])
    ud.ud_gather_status(sb.cuda_stream)
    with pytest.raises(ud.UdIndexError) as e:
        ud.ud_gather_status(sa.cuda_stream)
    assert e.value.pos == 777
    ud.ud_gather_status(sa.cuda_stream)
    assert np.array_equal(outs[1].cpu().numpy().view(np.uint32), oracle_bits(t.numpy(), good, oracle.F32))
    # B's bad gather is in flight while A's record is read and cleared: B's error is not lost
    launch(sa, d_a, outs[0])
    for _ in range(3):
        launch(sb, d_good, outs[1])
    launch(sb, d_b, outs[1])
    with pytest.raises(ud.UdIndexError) as e:
        ud.ud_gather_status(sa.cuda_stream)
    assert e.value.pos == 777
    ud.ud_gather_status(sa.cuda_stream)
    with pytest.raises(ud.UdIndexError) as e:
        ud.ud_gather_status(sb.cuda_stream)
    assert e.value.pos == M - 3
    for st in (sa, sb):
        ud.ud_gather_status(st.cuda_stream)
    # a stream that never launched anything has nothing to report
    ud.ud_gather_status(torch.cuda.Stream().cuda_stream)
    t.free()


def test_more_streams_than_error_slots(ud):
    # streams beyond the per-device slot table share one record; results and reports stay correct
    N, D, M = 2000, 64, 1500
    t = make_table(ud, N, D, ud.UD_F32, 68)
    idx = workloads.indices_uniform(69, M, N)
    want = oracle_bits(t.numpy(), idx, oracle.F32)
    didx = torch.from_numpy(idx).cuda()
    bad = idx.copy()
    bad[5] = N
    dbad = torch.from_numpy(bad).cuda()
    out = torch.empty((M, D), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    from conftest import RawStreams
    streams = RawStreams(140)
    # used one after the other, each followed by its status call: slots are handed on, every stream has its own record
    for st in streams.handles[:70]:
        ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, out.data_ptr(), st)
        ud.ud_gather_status(st)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), want)
    # 70 streams with work outstanding at once: those beyond the table share one record
    outs = torch.zeros((70, M, D), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    for k, st in enumerate(streams.handles[70:]):
        ids = dbad if k in (3, 69) else didx
        ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, ids.data_ptr(), ud.UD_I64, M, outs[k].data_ptr(), st)
    reported = 0
    for k, st in enumerate(streams.handles[70:]):
        try:
            ud.ud_gather_status(st)
        except ud.UdIndexError as e:
            assert e.pos == 5
            reported += 1
    assert 1 <= reported <= 2 + 7         # stream 3 reports its own; stream 69's may surface on any sharer of the common record
    got = outs.cpu().numpy().view(np.uint32)
    for k in range(70):
        if k not in (3, 69):
            assert np.array_equal(got[k], want), k
    for st in streams.handles[70:]:
        ud.ud_gather_status(st)
    streams.close()
    t.free()


def test_error_slots_change_hands_between_host_threads(ud):
    # four host threads, each driving its own 40 streams (160 streams for 63 slots): every launch is followed by its
    # status call, so slots are idle most of the time and are handed from stream to stream across threads all
    # the time; each report must be exactly what that stream was given
    import threading
    N, D, M = 3000, 64, 2000
    t = make_table(ud, N, D, ud.UD_F32, 71)
    idx = workloads.indices_uniform(72, M, N)
    want = oracle_bits(t.numpy(), idx, oracle.F32)
    bad_positions = (0, 777, M - 1)
    d_ids = [torch.from_numpy(idx).cuda()]
    for pos in bad_positions:
        b = idx.copy()
        b[pos] = N + pos
        d_ids.append(torch.from_numpy(b).cuda())
    n_threads, per_thread, rounds = 4, 40, 3
    outs = [torch.zeros((M, D), dtype=torch.float32, device="cuda") for _ in range(n_threads)]
    torch.cuda.synchronize()
    from conftest import RawStreams
    streams = RawStreams(n_threads * per_thread)
    failures = []

    def drive(k):
        try:
            mine = streams.handles[k * per_thread:(k + 1) * per_thread]
            for r in range(rounds):
                for j, st in enumerate(mine):
                    which = (k + 3 * j + r) % 4                 # 0: clean, else a bad ID at bad_positions[which - 1]
                    ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, d_ids[which].data_ptr(), ud.UD_I64, M, outs[k].data_ptr(), st)
                    try:
                        ud.ud_gather_status(st)
                        got = None
                    except ud.UdIndexError as e:
                        got = e.pos
                    expect = None if which == 0 else bad_positions[which - 1]
                    if got != expect:
                        failures.append((k, r, j, which, got))
                    if which == 0 and j % 8 == 0 and not np.array_equal(outs[k].cpu().numpy().view(np.uint32), want):
                        failures.append((k, r, j, "data"))
        except Exception as e:                                   # noqa: BLE001 - reported by the main thread
            failures.append((k, repr(e)))

    threads = [threading.Thread(target=drive, args=(k,)) for k in range(n_threads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not failures, failures[:5]
    for st in streams.handles:
        ud.ud_gather_status(st)
    streams.close()
    t.free()


def test_gathers_captured_in_a_hip_graph_replay_correctly(ud):
    # a launch-bound inner loop (several small gathers) captured once and replayed with new IDs each time;
    # the first eager call is what allocates the library's error word, so it runs before capture
    N, M = 20_000, 3001
    widths = (16, 100, 602)
    t = make_table(ud, N, 602, ud.UD_F32, 64)
    didx = torch.zeros(M, dtype=torch.int64, device="cuda")
    outs = {D: torch.zeros((M, D), dtype=torch.float32, device="cuda") for D in widths}
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for D in widths:                                           # eager warm-up on the capture stream
            ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, outs[D].data_ptr(), side.cuda_stream)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        cs = torch.cuda.current_stream().cuda_stream
        for D in widths:
            ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, outs[D].data_ptr(), cs)
    for rep in range(4):
        idx = workloads.indices_uniform(65 + rep, M, N)
        didx.copy_(torch.from_numpy(idx))
        torch.cuda.synchronize()                                   # the program's own eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        ud.ud_gather_status(side.cuda_stream)                      # the record of the stream the gathers were captured on
        for D in widths:
            view = np.ascontiguousarray(t.numpy().ravel()[: N * D].reshape(N, D))
            assert np.array_equal(outs[D].cpu().numpy().view(np.uint32), oracle_bits(view, idx, oracle.F32)), (rep, D)
    # a bad ID met during a replay is reported on that stream, and only there
    idx = workloads.indices_uniform(70, M, N)
    idx[1234] = N
    didx.copy_(torch.from_numpy(idx))
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    ud.ud_gather_status(None)
    with pytest.raises(ud.UdIndexError) as e:
        ud.ud_gather_status(side.cuda_stream)
    assert e.value.pos == 1234
    ud.ud_gather_status(side.cuda_stream)                          # cleared
    t.free()



@pytest.mark.parametrize("D", [1, 2, 3, 4, 5, 16, 25, 100, 129, 255, 256, 257, 513, 602, 603, 1031, 4099])
def test_device_resident_table_widths(ud, D):
    # an HBM-resident table takes the destination-aligned kernel by default; the source-aligned one
    # (small lane groups, two rows in flight, streaming stores) must give the same bits.  Output
    # offsets 0..3 elements put the output in every alignment class of the 16-byte chunk grid.
    N, M = 4001, 3777
    host = make_table(ud, N, D, ud.UD_F32, 900 + D)
    dev = host.to_device()
    idx = workloads.indices_uniform(90, M, N)
    idx[:2] = [0, N - 1]
    want = oracle_bits(host.numpy(), idx, oracle.F32)
    for off in range(4):
        assert np.array_equal(run_gather(ud, dev, idx, ud.UD_F32, out_offset_elems=off), want), (D, off)
    got = run_gather(ud, dev, idx, ud.UD_F32, ud.ud_tuning(0, 0, 2, 0, ud.UD_TUNE_NT_STORE), out_offset_elems=D % 4)
    assert np.array_equal(got, want), D
    dev.free()
    host.free()


@pytest.mark.parametrize("P", [1, 2, 4])
def test_destination_aligned_kernel_every_instantiation(ud, P):
    # every (dtype, chunks per lane, streaming or plain store) form of the destination-aligned kernel, on host and
    # HBM tables, for widths below, at and above one wavefront tile, with int32 and int64 IDs and a capped grid
    N, M = 1201, 1103
    cases = [(ud.UD_F32, ud.UD_F32, 77), (ud.UD_F32, ud.UD_F32, 2), (ud.UD_F32, ud.UD_F32, 1030),
             (ud.UD_F16, ud.UD_F16_TO_F32, 301), (ud.UD_F16, ud.UD_F16_TO_F32, 5), (ud.UD_F16, ud.UD_F16, 75),
             (ud.UD_F16, ud.UD_F16, 7), (ud.UD_F16, ud.UD_F16, 2051)]
    for elem, dtype, D in cases:
        t = make_table(ud, N, D, elem, 300 + D)
        d = t.to_device()
        for idt in (np.int64, np.int32):
            idx = workloads.indices_uniform(9, M, N, idt)
            idx[:2] = [0, N - 1]
            want = oracle_bits(t.numpy(), idx, dtype)
            for table in (t, d):
                for flags in (ud.UD_TUNE_DEST_ALIGNED, ud.UD_TUNE_DEST_ALIGNED | ud.UD_TUNE_NT_STORE):
                    for blocks in (0, 3):
                        for off in (0, 1, 3):
                            got = run_gather(ud, table, idx, dtype, ud.ud_tuning(0, P, 0, blocks, flags), out_offset_elems=off)
                            assert np.array_equal(got, want), (dtype, D, idt, table is d, flags, blocks, off)
        d.free()
        t.free()


def test_destination_aligned_kernel_reports_bad_ids_and_skips_their_rows(ud):
    N, D, M = 500, 602, 4000
    t = make_table(ud, N, D, ud.UD_F32, 22)
    d = t.to_device()
    idx = workloads.indices_uniform(23, M, N)
    for bad_positions, bad_values in (([3111, 1717, 2500], [N, -1, N + 5]), ([0], [-7]), ([M - 1], [2**40])):
        bad = idx.copy()
        bad[bad_positions] = bad_values
        out = torch.zeros((M, D), dtype=torch.float32, device="cuda")
        s = torch.cuda.current_stream().cuda_stream
        ud.ud_gather(d.device_ptr, N, D, ud.UD_F32, torch.from_numpy(bad).cuda().data_ptr(), ud.UD_I64, M, out.data_ptr(), s)
        with pytest.raises(ud.UdIndexError) as e:
            ud.ud_gather_status(s)
        assert e.value.pos == min(bad_positions)
        host = out.cpu().numpy()
        good = np.ones(M, dtype=bool)
        good[bad_positions] = False
        assert np.array_equal(host[good], t.numpy()[idx[good]])
        assert (host[~good] == 0).all()                              # bad rows are left unwritten, neighbours intact
    d.free()
    t.free()


@pytest.mark.parametrize("D", [3, 301, 602])
def test_device_resident_fp16_table(ud, D):
    N, M = 3001, 2500
    host = make_table(ud, N, D, ud.UD_F16, 950 + D)
    dev = host.to_device()
    idx = workloads.indices_uniform(91, M, N, np.int32)
    for dtype in (ud.UD_F16, ud.UD_F16_TO_F32):
        assert np.array_equal(run_gather(ud, dev, idx, dtype), oracle_bits(host.numpy(), idx, dtype)), (D, dtype)
    dev.free()
    host.free()


def test_torch_convenience_wrapper(ud):
    # table.py only marshals: pointers from torch tensors, output allocation, stream
    N, D, M = 5000, 100, 3001
    t = make_table(ud, N, D, ud.UD_F32, 80)
    idx_np = workloads.indices_uniform(81, M, N)
    idx = torch.from_numpy(idx_np).cuda()
    out = ud.gather(t, idx, check=True)
    assert out.shape == (M, D) and out.dtype == torch.float32 and out.is_cuda
    assert np.array_equal(out.cpu().numpy().view(np.uint32), oracle_bits(t.numpy(), idx_np, oracle.F32))
    pre = torch.empty((M, D), dtype=torch.float32, device="cuda")
    assert ud.gather(t, idx.to(torch.int32), out=pre, check=True) is pre
    assert torch.equal(pre, out)
    pinned_ids = torch.from_numpy(idx_np).pin_memory()            # the ID list left in pinned host memory: no copy
    assert torch.equal(ud.gather(t, pinned_ids, check=True), out)
    bad = idx.clone()
    bad[7] = N
    with pytest.raises(ud.UdIndexError):
        ud.gather(t, bad, check=True)
    h = make_table(ud, N, D, ud.UD_F16, 82)
    o16 = ud.gather(h, idx, check=True)
    o32 = ud.gather(h, idx, widen=True, check=True)
    assert o16.dtype == torch.float16 and o32.dtype == torch.float32
    assert np.array_equal(o32.cpu().numpy().view(np.uint32), oracle_bits(h.numpy(), idx_np, oracle.F16_TO_F32))
    assert torch.equal(o16.float(), o32)
    with pytest.raises(ValueError):
        t.to_device().numpy()
    h.free()
    t.free()


# ---- padded tables: row pitch rounded up to 128 bytes ----

@pytest.mark.parametrize("elem_name,dtype_name,D", [("UD_F32", "UD_F32", 1), ("UD_F32", "UD_F32", 100), ("UD_F32", "UD_F32", 602),
                                                     ("UD_F32", "UD_F32", 128), ("UD_F16", "UD_F16_TO_F32", 602),
                                                     ("UD_F16", "UD_F16", 301)])
def test_padded_table(ud, elem_name, dtype_name, D):
    elem, dtype = getattr(ud, elem_name), getattr(ud, dtype_name)
    N, M = 4001, 5003
    t = ud.Table(N, D, elem, ud.UD_TABLE_PAD_ROWS)
    per_line = 128 // t.elem_bytes
    assert t.pitch == -(-D // per_line) * per_line and t.pitch >= D and t.device_ptr % 128 == 0
    # fill data and padding alike, then poison the padding: it must never reach the output
    if elem == ud.UD_F32:
        workloads.fill_uniform_f32(t.host_ptr, 40, N * t.pitch)
    else:
        workloads.fill_normal_f16(t.host_ptr, 40, N * t.pitch)
    storage = np.frombuffer((ctypes.c_char * t.nbytes).from_address(t.host_ptr),
                            dtype=np.uint32 if elem == ud.UD_F32 else np.uint16).reshape(N, t.pitch)
    storage[:, D:] = 0xFFFF
    idx = workloads.indices_uniform(41, M, N)
    idx[:2] = [0, N - 1]
    obytes = 2 if dtype == ud.UD_F16 else 4
    want = np.empty((M, D), dtype=np.uint16 if obytes == 2 else np.uint32)
    oracle.gather_raw(t.host_ptr, N, D, dtype, idx, want, pitch=t.pitch)
    if dtype != ud.UD_F16_TO_F32:                                  # bit copies: numpy on the padded storage agrees
        assert np.array_equal(np.take(storage, idx, axis=0)[:, :D], want)
    for table in (t, t.to_device()):
        buf = torch.full(((M * D + 64) * obytes,), CANARY, dtype=torch.uint8, device="cuda")
        didx = torch.from_numpy(idx).cuda()
        s = torch.cuda.current_stream().cuda_stream
        ud.ud_gather_pitched(table.device_ptr, N, D, table.pitch, dtype, didx.data_ptr(), ud.UD_I64, M, buf.data_ptr(), s)
        ud.ud_gather_status(s)
        host = buf.cpu().numpy()
        assert (host[M * D * obytes:] == CANARY).all()
        assert np.array_equal(host[: M * D * obytes].view(want.dtype).reshape(M, D), want), (D, table.host_ptr != 0)
    # the hot-row cache works on padded tables too
    c = ud.Cache(t, np.arange(0, N, 2, dtype=np.int64))
    assert np.array_equal(run_cached(ud, c, dtype, idx, D), want)
    c.free()
    t.free()


def test_padded_table_through_the_torch_wrapper(ud):
    N, D, M = 3000, 602, 2000
    t = ud.Table(N, D, ud.UD_F32, ud.UD_TABLE_PAD_ROWS)
    assert t.pitch == 608
    data = workloads.uniform_f32(42, N, D)
    t.numpy()[:] = data                                           # the [N, D] window of the padded storage
    idx_np = workloads.indices_uniform(43, M, N)
    out = ud.gather(t, torch.from_numpy(idx_np).cuda(), check=True)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), oracle.gather(data, idx_np).view(np.uint32))
    t.free()
