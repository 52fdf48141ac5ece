"""Seeded random sweep of shapes, alignments, dtypes and launch shapes: GPU vs oracle, bit for bit.

Every case is small; together they cover combinations no hand-written case names (odd widths with
odd base offsets, tiny M, group sizes that do not match the width, cached and padded tables, ...)."""
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


SHAPES = [(1, 1), (2, 1), (4, 1), (1, 2), (2, 2), (1, 3), (2, 3), (1, 4), (2, 4)]


def test_random_gathers(ud):
    rng = np.random.default_rng(20260101)
    s = torch.cuda.current_stream().cuda_stream
    for case in range(160):
        elem = ud.UD_F32 if rng.random() < 0.6 else ud.UD_F16
        esz = 4 if elem == ud.UD_F32 else 2
        dtype = elem if elem == ud.UD_F32 else (ud.UD_F16 if rng.random() < 0.5 else ud.UD_F16_TO_F32)
        obytes = 2 if dtype == ud.UD_F16 else 4
        D = int(rng.choice([1, 2, 3, 5, 7, 8, 13, 16, 31, 32, 33, 63, 64, 65, 100, 127, 129, 255, 257, 301, 602, 777, 1025]))
        N = int(rng.integers(1, 3000))
        M = int(rng.integers(1, 4000))
        shift = int(rng.integers(0, 8))                       # table base offset in elements: any alignment class
        big = ud.Table(N + 1, D + 8, elem)
        n_el = (N + 1) * (D + 8)
        if elem == ud.UD_F32:
            workloads.fill_uniform_f32(big.host_ptr, case, n_el)
        else:
            workloads.fill_normal_f16(big.host_ptr, case, n_el)
        flat = np.frombuffer((__import__("ctypes").c_char * big.nbytes).from_address(big.host_ptr),
                             dtype=np.uint32 if esz == 4 else np.uint16)
        view = np.ascontiguousarray(flat[shift:shift + N * D].reshape(N, D))
        idt = np.int64 if rng.random() < 0.5 else np.int32
        idx = rng.integers(0, N, size=M).astype(idt)
        want = oracle.gather(view, idx, {ud.UD_F32: oracle.F32, ud.UD_F16: oracle.F16, ud.UD_F16_TO_F32: oracle.F16_TO_F32}[dtype])
        want = want.view(np.uint16 if obytes == 2 else np.uint32)
        u, p = SHAPES[int(rng.integers(0, len(SHAPES)))]
        lanes = int(2 ** rng.integers(0, 7))
        flags = int(rng.choice([0, 0, ud.UD_TUNE_NT_STORE, ud.UD_TUNE_NT_STORE, ud.UD_TUNE_DEST_ALIGNED,
                                ud.UD_TUNE_DEST_ALIGNED | ud.UD_TUNE_NT_STORE, ud.UD_TUNE_ELEMENTWISE,
                                ud.UD_TUNE_ELEMENTWISE | ud.UD_TUNE_CIRCULAR_SHIFT, ud.UD_TUNE_SHARE_GPU]))
        blocks = int(rng.choice([0, 1, 3, 64]))
        tun = None if rng.random() < 0.25 else ud.ud_tuning(lanes, p, u, blocks, flags)
        if tun is not None and (flags & ud.UD_TUNE_SHARE_GPU):
            tun = ud.ud_tuning(0, 0, 0, blocks, flags)
        if tun is not None and (flags & ud.UD_TUNE_DEST_ALIGNED):
            tun = ud.ud_tuning(0, int(rng.choice([0, 1, 2, 4])), 0, blocks, flags)
        out_shift = int(rng.integers(0, 5))
        buf = torch.full(((M * D + out_shift + 32) * obytes,), 0x5A, dtype=torch.uint8, device="cuda")
        didx = torch.from_numpy(idx).cuda()
        tag = (case, D, N, M, shift, dtype, lanes, u, p, flags, blocks, out_shift, tun is None)
        print("gather case", tag, flush=True)
        in_hbm = rng.random() < 0.3
        src_table = big.to_device() if in_hbm else big
        ud.ud_gather_tuned(src_table.device_ptr + shift * esz, N, D, dtype, didx.data_ptr(),
                           ud.UD_I64 if idt == np.int64 else ud.UD_I32, M, buf.data_ptr() + out_shift * obytes, s, tun)
        ud.ud_gather_status(s)
        host = buf.cpu().numpy()
        lo, hi = out_shift * obytes, (out_shift + M * D) * obytes
        assert (host[:lo] == 0x5A).all() and (host[hi:] == 0x5A).all(), tag
        assert np.array_equal(host[lo:hi].view(want.dtype).reshape(M, D), want), tag
        if in_hbm:
            src_table.free()
        big.free()


def test_random_scatters(ud):
    rng = np.random.default_rng(20260202)
    s = torch.cuda.current_stream().cuda_stream
    shapes = [(1, 1), (2, 1), (4, 1), (1, 2), (2, 2), (1, 3), (1, 4)]
    for case in range(80):
        esz = 4 if rng.random() < 0.6 else 2
        dtype = ud.UD_F32 if esz == 4 else ud.UD_F16
        D = int(rng.choice([1, 2, 3, 5, 8, 13, 16, 33, 64, 65, 100, 129, 257, 301, 602, 1025]))
        N = int(rng.integers(2, 2500))
        M = int(rng.integers(1, N + 1))
        shift = int(rng.integers(0, 8))
        big = ud.Table(N + 1, D + 8, dtype)
        storage = np.frombuffer((__import__("ctypes").c_char * big.nbytes).from_address(big.host_ptr),
                                dtype=np.uint32 if esz == 4 else np.uint16)
        storage[:] = rng.integers(0, 2 ** (8 * esz), size=storage.size, dtype=np.uint64).astype(storage.dtype)
        want_all = storage.copy()
        idt = np.int64 if rng.random() < 0.5 else np.int32
        idx = rng.permutation(N)[:M].astype(idt)
        src = rng.integers(0, 2 ** (8 * esz), size=(M, D), dtype=np.uint64).astype(storage.dtype)
        win = want_all[shift:shift + N * D].reshape(N, D)     # a view: the oracle writes into want_all
        oracle.scatter(win, idx, src)
        u, p = shapes[int(rng.integers(0, len(shapes)))]
        tun = None if rng.random() < 0.3 else ud.ud_tuning(int(2 ** rng.integers(0, 7)), p, u, int(rng.choice([0, 1, 5])), 0)
        if rng.random() < 0.35:                                  # the source-aligned kernel
            tun = ud.ud_tuning(0, int(rng.choice([0, 1, 2, 4])), 0, int(rng.choice([0, 1, 5])),
                               ud.UD_TUNE_FLAT_SOURCE | (ud.UD_TUNE_NT_STORE if rng.random() < 0.5 else 0))
        tag = (case, D, N, M, shift, esz, tun is None)
        print("scatter case", tag, flush=True)
        dsrc = torch.from_numpy(src.view(np.int32 if esz == 4 else np.int16)).cuda()
        didx = torch.from_numpy(idx).cuda()
        ud.ud_scatter(big.device_ptr + shift * esz, N, D, dtype, didx.data_ptr(),
                      ud.UD_I64 if idt == np.int64 else ud.UD_I32, M, dsrc.data_ptr(), s, tun)
        ud.ud_gather_status(s)
        assert np.array_equal(storage, want_all), tag            # the rows named, and nothing else, changed
        big.free()
