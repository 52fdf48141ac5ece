"""ud_gather_noalloc -- the gather for callers that must not allocate -- against ud_gather, through the C ABI.

Its kernels are ud_gather's; what differs is where the ID-error slots live (a static device array
instead of an allocated table).  Outputs must be bit-identical to ud_gather's (which the other tests
hold against the oracle), on two calls in a row, the second with a smaller input, and ID errors must
be reported the same way.  Collected last; passes alone in a fresh process and after the other tests.
"""
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


def run(ud, fn, table, idx_np, dtype, stream):
    M = idx_np.size
    obytes = 2 if dtype == ud.UD_F16 else 4
    buf = torch.full(((M * table.D + 64) * obytes,), CANARY, dtype=torch.uint8, device="cuda")
    idx = torch.from_numpy(idx_np).cuda()
    torch.cuda.synchronize()
    fn(table.device_ptr, table.N, table.D, dtype, idx.data_ptr(), ud.UD_I64 if idx_np.dtype == np.int64 else ud.UD_I32,
       M, buf.data_ptr(), stream)
    ud.ud_gather_status(stream)
    host = buf.cpu().numpy()
    assert (host[M * table.D * obytes:] == CANARY).all(), "wrote past the output"
    return host[: M * table.D * obytes].view(np.uint16 if obytes == 2 else np.uint32).reshape(M, table.D)


@pytest.mark.parametrize("elem_name,dtype_name,D", [("UD_F32", "UD_F32", 602), ("UD_F32", "UD_F32", 100), ("UD_F32", "UD_F32", 16),
                                                     ("UD_F16", "UD_F16_TO_F32", 301), ("UD_F16", "UD_F16", 75)])
def test_noalloc_gather_equals_ud_gather_on_two_calls_the_second_smaller(ud, elem_name, dtype_name, D):
    elem, dtype = getattr(ud, elem_name), getattr(ud, dtype_name)
    N = 20_011
    host = ud.Table(N, D, elem)
    (workloads.fill_uniform_f32 if elem == ud.UD_F32 else workloads.fill_normal_f16)(host.host_ptr, 7000 + D, N * D)
    dev = host.to_device()
    side = torch.cuda.Stream()
    for table in (host, dev):
        for stream in (torch.cuda.current_stream().cuda_stream, side.cuda_stream):
            for M, idt in ((30_011, np.int64), (4_097, np.int32)):          # the second call is the smaller one
                idx = workloads.indices_uniform(7100 + M, M, N, idt)
                idx[:2] = [0, N - 1]
                got = run(ud, ud.ud_gather_noalloc, table, idx, dtype, stream)
                want = run(ud, ud.ud_gather, table, idx, dtype, stream)
                assert np.array_equal(got, want), (D, table is dev, M)
                # ... which in turn is the oracle's result
                o = oracle.gather(host.numpy(), idx, {ud.UD_F32: oracle.F32, ud.UD_F16: oracle.F16,
                                                      ud.UD_F16_TO_F32: oracle.F16_TO_F32}[dtype])
                assert np.array_equal(got, o.view(got.dtype))
    dev.free()
    host.free()


def test_noalloc_gather_reports_bad_ids_per_stream_and_clears_them(ud):
    N, D, M = 5_000, 128, 9_001
    t = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(t.host_ptr, 7200, N * D)
    good = workloads.indices_uniform(7201, M, N)
    bad = good.copy()
    bad[[4321, 17]] = [N, -1]
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    d_good, d_bad = torch.from_numpy(good).cuda(), torch.from_numpy(bad).cuda()
    out = [torch.zeros((M, D), dtype=torch.float32, device="cuda") for _ in range(2)]
    torch.cuda.synchronize()
    ud.ud_gather_noalloc(t.device_ptr, N, D, ud.UD_F32, d_bad.data_ptr(), ud.UD_I64, M, out[0].data_ptr(), sa.cuda_stream)
    ud.ud_gather_noalloc(t.device_ptr, N, D, ud.UD_F32, d_good.data_ptr(), ud.UD_I64, M, out[1].data_ptr(), sb.cuda_stream)
    ud.ud_gather_status(sb.cuda_stream)                                  # stream B saw nothing bad
    with pytest.raises(ud.UdIndexError) as e:
        ud.ud_gather_status(sa.cuda_stream)
    assert e.value.pos == 17
    ud.ud_gather_status(sa.cuda_stream)                                  # read once, cleared
    host = out[0].cpu().numpy()
    ok = np.ones(M, dtype=bool)
    ok[[4321, 17]] = False
    assert np.array_equal(host[ok], t.numpy()[bad[ok]]) and (host[~ok] == 0).all()
    assert np.array_equal(out[1].cpu().numpy(), t.numpy()[good])
    # the slot keeps what earlier calls left until it is read: two bad calls, one report of the smaller position
    ud.ud_gather_noalloc(t.device_ptr, N, D, ud.UD_F32, d_bad.data_ptr(), ud.UD_I64, M, out[0].data_ptr(), sa.cuda_stream)
    ud.ud_gather_noalloc(t.device_ptr, N, D, ud.UD_F32, d_bad.data_ptr(), ud.UD_I64, 18, out[0].data_ptr(), sa.cuda_stream)
    with pytest.raises(ud.UdIndexError) as e:
        ud.ud_gather_status(sa.cuda_stream)
    assert e.value.pos == 17
    ud.ud_gather_status(sa.cuda_stream)
    t.free()


def test_noalloc_gather_refuses_a_64th_stream_with_a_clear_error(ud):
    N, D, M = 1_000, 64, 777
    t = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(t.host_ptr, 7300, N * D)
    idx = workloads.indices_uniform(7301, M, N)
    didx = torch.from_numpy(idx).cuda()
    out = torch.zeros((M, D), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    from conftest import RawStreams
    raw = RawStreams(140)
    streams = raw.handles[70:]
    # one after the other, each followed by its status call: slots are handed on, nobody is refused
    for st in raw.handles[:70]:
        ud.ud_gather_noalloc(t.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, out.data_ptr(), st)
        ud.ud_gather_status(st)
        assert np.array_equal(out.cpu().numpy(), t.numpy()[idx])
    # 70 streams with work outstanding at once: the fixed array has 63 slots
    refused, accepted = 0, []
    for st in streams:
        rc = ud.binding.raw_status("ud_gather_noalloc", t.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M,
                                   out.data_ptr(), st)
        if rc == ud.UD_OK:
            accepted.append(st)
        else:
            refused += 1
            assert rc == ud.UD_ERR_UNSUPPORTED and "static error slots" in ud.ud_last_hip_error()
    assert 70 - 63 <= refused < 70 and accepted[0] == streams[0]          # slots held by other live streams may add to it
    for st in accepted:
        ud.ud_gather_status(st)
    assert np.array_equal(out.cpu().numpy(), t.numpy()[idx])
    # streams that hold a slot keep working, and so does the allocating entry point on any stream
    ud.ud_gather_noalloc(t.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, out.data_ptr(), streams[0])
    ud.ud_gather_status(streams[0])
    ud.ud_gather(t.device_ptr, N, D, ud.UD_F32, didx.data_ptr(), ud.UD_I64, M, out.data_ptr(), streams[-1])
    ud.ud_gather_status(streams[-1])
    assert np.array_equal(out.cpu().numpy(), t.numpy()[idx])
    raw.close()
    t.free()
