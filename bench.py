#!/usr/bin/env python3
"""Benchmark of the zero-copy feature-row gather on one MI355X.

Workload (default): the gather microbenchmark sweep -- a host-pinned fp32 table
of 4,000,000 x D for D in {16, 64, 100, 128, 256, 602} (values uniform[-1,1),
seed 1), 1,000,000 int64 row IDs drawn uniformly with replacement.  One *step*
is one pass of the whole hot path over one batch: six gathers, one per width,
each from pinned host memory straight into HBM.  Table, ID lists and output
are resident (table in pinned host memory -- that is the point -- IDs and
output in HBM) before the timed region starts.

Prints ONE JSON line:
  value     = useful bytes crossing the host link / time, GB/s (1e9), all widths
  roofline  = the dominant kernel (the D=602 gather) against the host-link peak,
              i.e. the best pinned hipMemcpy H2D rate measured in this same run
  roofline_hbm = the device-resident variant (table in HBM) vs 8 TB/s
  cpu_baseline = the CPU oracle timed on this machine's host cores
  cpu_centric  = the path the paper argues against (CPU gather -> pinned staging
                 -> hipMemcpyAsync), plain and double-buffered
  configs      = the other benchmark configurations, few repetitions each: single
                 gather, GraphSAGE-style minibatches, the large host table (with
                 the record of what the host would pin) and its HBM slice, the
                 fp16 odd-width table with the fused upcast
  experiments  = the paper's alignment sweep (Figure 7) and size grid (Figure 6),
                 the write direction, the hot-row cache, overlap with a consumer
Every entry of configs / experiments carries its own parity_spot_check against
the oracle.  `--workload NAME` runs one of them alone, with full repetitions, as
a line of its own; `--headline-only` stops after the headline.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WIDTHS = (16, 64, 100, 128, 256, 602)
N_ROWS = 4_000_000
M_ROWS = 1_000_000
TABLE_SEED = 1
HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak


def _load_baseline_lib(ud):
    path = os.path.join(os.path.dirname(ud.LIB_PATH), "libud_baseline.so")
    bl = ctypes.CDLL(path)
    dp = ctypes.POINTER(ctypes.c_double)
    bl.udb_h2d_peak.argtypes = [ctypes.c_size_t, ctypes.c_int, dp, dp]
    bl.udb_d2d_peak.argtypes = [ctypes.c_size_t, ctypes.c_int, dp, dp]
    bl.udb_d2h_peak.argtypes = [ctypes.c_size_t, ctypes.c_int, dp, dp]
    bl.udb_plain_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    bl.udb_cpu_centric_create.argtypes = [ctypes.c_size_t, ctypes.POINTER(ctypes.c_void_p)]
    bl.udb_cpu_centric_destroy.argtypes = [ctypes.c_void_p]
    bl.udb_cpu_centric_gather.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                          ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, dp, dp, dp]
    return bl


def _read_traffic_note(ud, table_ptr, key, plan_key):
    """Fabric traffic (bytes per launch) of the dominant kernel, measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE and kept in the committed counter summary.  The summary names the launch shape it was
    measured on; if ud_gather_plan picks another shape today the figure no longer describes this build and
    None is returned with the reason."""
    path = os.path.join(ROOT, "profiles", "gather_f32_D602_traffic.txt")
    if not os.path.exists(path):
        return None, "profiles/gather_f32_D602_traffic.txt is absent"
    vals = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.strip().split("=", 1)
            vals[k] = v
    p = ud.ud_gather_plan(table_ptr, 602, ud.UD_F32)
    now = f"lanes={p.lanes_per_row},chunks={p.chunks_per_lane},rows={p.rows_in_flight},max_blocks={p.max_blocks},flags={p.flags}"
    if vals.get(plan_key) != now:
        return None, f"measured on plan [{vals.get(plan_key)}], this build launches [{now}]: re-measure"
    if key not in vals:
        return None, f"{key} missing from the summary"
    return float(vals[key]), None


def _host_topology():
    """Sockets and NUMA nodes of the host, as far as /proc and /sys tell."""
    info = {}
    try:
        phys = {line.split(":")[1].strip() for line in open("/proc/cpuinfo") if line.startswith("physical id")}
        info["sockets"] = len(phys) or None
        info["cpu_model"] = next((line.split(":", 1)[1].strip() for line in open("/proc/cpuinfo")
                                  if line.startswith("model name")), None)
        nodes = [d for d in os.listdir("/sys/devices/system/node") if d.startswith("node") and d[4:].isdigit()]
        info["numa_nodes"] = len(nodes) or None
        info["cpus_online"] = os.cpu_count()
    except OSError:
        pass
    return info


def _stats(ms):
    ms = sorted(ms)
    return {"median_ms": round(ms[len(ms) // 2], 4), "min_ms": round(ms[0], 4), "reps": len(ms)}


def _itype(ud, t):
    import torch
    return ud.UD_I64 if t.dtype == torch.int64 else ud.UD_I32


def _kernel_times(ud, torch, tptr, N, D, dtype, id_tensors, out, warm, tuning=None):
    """Kernel-only time (HIP events on the launch stream) of one gather per ID tensor; the first `warm` are untimed."""
    stream = torch.cuda.current_stream().cuda_stream
    ev = []
    for k, ids in enumerate(id_tensors):
        if k >= warm:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        ud.ud_gather_tuned(tptr, N, D, dtype, ids.data_ptr(), _itype(ud, ids), ids.numel(), out.data_ptr(), stream, tuning)
        if k >= warm:
            e1.record()
            ev.append((e0, e1))
    torch.cuda.synchronize()
    ud.ud_gather_status(stream)
    return [a.elapsed_time(b) for a, b in ev]


def _wall_times(ud, torch, tptr, N, D, dtype, ids_pinned, out, warm, ids_stay_in_host=False):
    """Call-to-sync wall time per gather INCLUDING the host->device copy of the ID list (pinned source).
    ids_stay_in_host: no copy, the kernel reads the ID list from pinned host memory as it reads the rows."""
    stream = torch.cuda.current_stream()
    dst = torch.empty(max(t.numel() for t in ids_pinned), dtype=ids_pinned[0].dtype, device="cuda")
    ms = []
    for k, ids in enumerate(ids_pinned):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        d = ids if ids_stay_in_host else dst[: ids.numel()]
        if not ids_stay_in_host:
            d.copy_(ids, non_blocking=True)
        ud.ud_gather(tptr, N, D, dtype, d.data_ptr(), _itype(ud, d), ids.numel(), out.data_ptr(), stream.cuda_stream)
        stream.synchronize()
        if k >= warm:
            ms.append((time.perf_counter() - t0) * 1e3)
    ud.ud_gather_status(stream.cuda_stream)
    return ms


def _cpu_centric(bl, ctx, table_host_ptr, row_bytes, ids_np, out_ptr, threads, slices=1):
    a, b, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    rc = bl.udb_cpu_centric_gather(ctx, table_host_ptr, row_bytes, ids_np.ctypes.data, ids_np.size, out_ptr,
                                   threads, slices, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    if rc != 0:
        raise RuntimeError(f"cpu-centric baseline failed ({rc})")
    return a.value * 1e3


def _h2d_rate(bl, nbytes, reps=10):
    best, med = ctypes.c_double(), ctypes.c_double()
    if bl.udb_h2d_peak(max(int(nbytes), 4096), reps, ctypes.byref(best), ctypes.byref(med)) != 0:
        raise RuntimeError("hipMemcpy rate measurement failed")
    return best.value


class Env:
    """What every workload needs: the libraries, the in-run host-link peak, repetition counts."""

    def __init__(self, ud, bl, workloads, torch, np, threads, ncores, K, W, no_cpu):
        self.ud, self.bl, self.workloads, self.torch, self.np = ud, bl, workloads, torch, np
        self.threads, self.ncores, self.K, self.W, self.no_cpu = threads, ncores, K, W, no_cpu
        self.dev = torch.device("cuda:0")
        self.h2d_peak = _h2d_rate(bl, 1 << 30)
        self._oracle = None

    @property
    def oracle(self):                      # the CPU oracle: spot checks and the cpu_baseline leg only
        if self._oracle is None:
            import oracle
            self._oracle = oracle
        return self._oracle

    def pinned(self, a):
        return self.torch.from_numpy(a).pin_memory()

    def spot_check(self, table, N, D, odtype, ids_np, out, n=2048, pitch=None):
        """Sampled output rows against the oracle, bit for bit."""
        np, torch = self.np, self.torch
        sample = np.sort(np.random.default_rng(0).choice(ids_np.size, min(n, ids_np.size), replace=False))
        got = out[: ids_np.size * D].view(ids_np.size, D)[torch.from_numpy(sample).to(self.dev)].cpu().numpy()
        want = np.empty((sample.size, D), dtype=np.uint32)
        kw = {} if pitch is None else {"pitch": pitch}
        self.oracle.gather_raw(table.host_ptr, N, D, odtype, np.ascontiguousarray(ids_np[sample]), want, **kw)
        return bool(np.array_equal(got.view(np.uint32), want))

    def event_times(self, launch, n, warm):
        """Kernel-only ms of launch(k) for k in warm..n-1 (HIP events on the current stream)."""
        torch = self.torch
        ev = []
        for k in range(n):
            if k >= warm:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            launch(k)
            if k >= warm:
                e1.record()
                ev.append((e0, e1))
        torch.cuda.synchronize()
        self.ud.ud_gather_status(torch.cuda.current_stream().cuda_stream)
        return [a.elapsed_time(b) for a, b in ev]


def _meminfo():
    out = {}
    try:
        for line in open("/proc/meminfo"):
            k, v = line.split(":", 1)
            if k in ("MemTotal", "MemAvailable"):
                out[k + "_kB"] = int(v.split()[0])
    except OSError:
        pass
    try:
        import resource
        soft, hard = resource.getrlimit(resource.RLIMIT_MEMLOCK)
        out["ulimit_l"] = "unlimited" if soft == resource.RLIM_INFINITY else soft
    except Exception:
        pass
    return out


#: the large host-resident table: the configuration's size first, then the largest round size that the MI355X
#: boxes this was developed on will pin (their hipHostMalloc refuses more than about 65.5 GiB in total)
LARGE_ROWS = (111_000_000, 62_500_000)


def alloc_large_table(ud, D):
    """The configuration's 111,000,000-row table, or the documented fallback; every refusal is recorded with
    what the host says about its memory.  Returns (table or None, rows, attempts)."""
    attempts = []
    for n in LARGE_ROWS:
        t0 = time.perf_counter()
        try:
            table = ud.Table(n, D, ud.UD_F32)
            attempts.append({"rows": n, "bytes": n * D * 4, "status": "UD_OK", "seconds": round(time.perf_counter() - t0, 2)})
            return table, n, attempts
        except ud.UdError as e:
            attempts.append({"rows": n, "bytes": n * D * 4, "GiB": round(n * D * 4 / 2**30, 1), "status": ud.ud_status_str(e.status),
                             "hip_error": ud.ud_last_hip_error(), "seconds": round(time.perf_counter() - t0, 2), **_meminfo()})
            if e.status != ud.UD_ERR_OOM:
                raise
    return None, 0, attempts


# ---------------------------------------------------------------------------------------------------------------
# The other configurations and experiments.  Each returns a dict with value (GB/s), ms_per_step, dtype, config and
# its own details; `quick` trims repetitions for the all-in-one default run.
# ---------------------------------------------------------------------------------------------------------------

def wl_single(env, quick=False):
    ud, torch, np, workloads, bl = env.ud, env.torch, env.np, env.workloads, env.bl
    K, W = (10 if quick else env.K), env.W
    N, D, M = 100_000, 128, 16_384
    table = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(table.host_ptr, 0, N * D)
    ids_np = [workloads.indices_uniform(workloads.IDX_STREAM + k, M, N) for k in range(K + W)]
    ids_dev = [torch.from_numpy(a).to(env.dev) for a in ids_np]
    out = torch.empty(M * D, dtype=torch.float32, device=env.dev)
    kern = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W)
    ok = env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out)
    wall = _wall_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, [env.pinned(a) for a in ids_np], out, W)
    nbytes = M * D * 4
    same_size = _h2d_rate(bl, nbytes, 20)
    ks, ws = _stats(kern), _stats(wall)
    # the same gather captured in a HIP graph and replayed: call-to-sync without the per-call launch path
    side = torch.cuda.Stream()
    gidx = ids_dev[0].clone()
    with torch.cuda.stream(side):
        ud.ud_gather(table.device_ptr, N, D, ud.UD_F32, gidx.data_ptr(), ud.UD_I64, M, out.data_ptr(), side.cuda_stream)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ud.ud_gather(table.device_ptr, N, D, ud.UD_F32, gidx.data_ptr(), ud.UD_I64, M, out.data_ptr(),
                     torch.cuda.current_stream().cuda_stream)
    gms = []
    for k in range(K + W):
        gidx.copy_(ids_dev[k])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        if k >= W:
            gms.append((time.perf_counter() - t0) * 1e3)
    ud.ud_gather_status(side.cuda_stream)
    ok = ok and env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out)
    table.free()
    gbps = nbytes / ks["median_ms"] / 1e6
    return {"value": gbps, "ms_per_step": ks["median_ms"], "dtype": "f32",
            "config": {"workload": "single gather: host-pinned fp32 100,000 x 128 (seed 0), 16,384 int64 IDs uniform with replacement"},
            "kernel_only": ks, "call_to_sync_incl_id_copy": ws, "wall_GBps": round(nbytes / ws["median_ms"] / 1e6, 2),
            "hip_graph_replay_call_to_sync": _stats(gms), "same_size_hipMemcpy_GBps": round(same_size, 2),
            "frac_of_same_size_hipMemcpy": round(gbps / same_size, 4), "rows_per_s": round(M / ks["median_ms"] * 1e3),
            "parity_spot_check": ok}


def _cpu_centric_legs(env, table, row_bytes, ids_np, out, cap_bytes, nbatch):
    bl, threads = env.bl, env.threads
    extra = {}
    ctx = ctypes.c_void_p()
    if bl.udb_cpu_centric_create(cap_bytes, ctypes.byref(ctx)) != 0:
        return None
    for name, th, sl in (("plain", threads, 1), ("double_buffered", threads, 4)):
        _cpu_centric(bl, ctx, table.host_ptr, row_bytes, ids_np[0], out.data_ptr(), th, sl)
        ms = [_cpu_centric(bl, ctx, table.host_ptr, row_bytes, a, out.data_ptr(), th, sl) for a in ids_np[:nbatch]]
        extra[name] = {"GBps": round(sum(a.size for a in ids_np[:nbatch]) * row_bytes / sum(ms) / 1e6, 2), "threads": th}
    bl.udb_cpu_centric_destroy(ctx)
    return extra


def _products_like_inputs(env, nb):
    ud, workloads = env.ud, env.workloads
    p = workloads.PRODUCTS_LIKE
    N, D = p["N"], p["D"]
    table = ud.Table(N, D, ud.UD_F32)
    workloads.fill_uniform_f32(table.host_ptr, 3, N * D)
    offsets, nbr = workloads.zipf_graph_csr(N, p["mean_degree"], p["dmin"], p["alpha"], 3)
    ids_np = [workloads.sample_csr(offsets, nbr, p["nseeds"], p["fanout"], 33, b) for b in range(nb)]
    return table, ids_np


def wl_graphsage(env, quick=False, inputs=None):
    ud, torch, np = env.ud, env.torch, env.np
    W = env.W
    nb = 20 if quick else 100
    table, ids_np = inputs if inputs else _products_like_inputs(env, nb)
    ids_np = ids_np[:nb]
    N, D = table.N, table.D
    ids_dev = [torch.from_numpy(a).to(env.dev) for a in ids_np]
    cap = max(a.size for a in ids_np)
    out = torch.empty(cap * D, dtype=torch.float32, device=env.dev)
    sorted_dev = [torch.from_numpy(np.sort(a)).to(env.dev) for a in ids_np]      # secondary: the same IDs in ascending order
    kern_sorted = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, sorted_dev[:W] + sorted_dev, out, W)
    del sorted_dev
    kern = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev[:W] + ids_dev, out, W)
    ok = env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out)
    pinned = [env.pinned(a) for a in ids_np]
    wall = _wall_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, pinned[:W] + pinned, out, W)
    total_bytes = sum(a.size for a in ids_np) * D * 4
    extra = None if env.no_cpu else _cpu_centric_legs(env, table, D * 4, ids_np, out, cap * D * 4, 5 if quick else 20)
    sizes = [a.size for a in ids_np]
    if not inputs:
        table.free()
    return {"value": total_bytes / sum(kern) / 1e6, "ms_per_step": sum(kern) / nb, "dtype": "f32",
            "config": {"workload": "GraphSAGE-style minibatch gather: 2,400,000 x 100 fp32 host-pinned table, Zipf power-law "
                                   f"CSR graph (mean degree 50), 1,024 seeds, fanout [25,10], de-duplicated; {nb} batches; "
                                   "one step = one batch", "unique_ids_per_batch": [min(sizes), max(sizes)], "batches": nb},
            "kernel_only": _stats(kern), "call_to_sync_incl_id_copy": _stats(wall),
            "sorted_ids_GBps": round(total_bytes / sum(kern_sorted) / 1e6, 2),
            "wall_GBps": round(total_bytes / sum(wall) / 1e6, 2), "rows_per_s": round(sum(sizes) / sum(kern) * 1e3),
            "cpu_centric": extra, "parity_spot_check": ok}


def _papers_like_inputs(env, nb):
    ud, workloads = env.ud, env.workloads
    p = workloads.PAPERS_LIKE
    t0 = time.perf_counter()
    table, N, attempts = alloc_large_table(ud, p["D"])
    if table is None:
        return None, 0, [], attempts, 0.0
    workloads.fill_uniform_f32(table.host_ptr, 4, N * p["D"])
    ready = time.perf_counter() - t0
    ids_np = [workloads.sample_procedural(N, p["degree"], p["alpha"], 4, p["nseeds"], p["fanout"], 44, b) for b in range(nb)]
    return table, N, ids_np, attempts, ready


def wl_large(env, quick=False, inputs=None):
    ud, torch, np, workloads = env.ud, env.torch, env.np, env.workloads
    W = env.W
    nb = 5 if quick else max(env.K, 5)
    table, N, ids_np, attempts, ready = inputs if inputs else _papers_like_inputs(env, nb)
    if table is None:
        return {"value": 0.0, "ms_per_step": 0.0, "dtype": "f32", "config": {"workload": "large host-resident table: not run"},
                "table_allocation_attempts": attempts, "parity_spot_check": False}
    ids_np = ids_np[:nb]
    D = table.D
    ids_dev = [torch.from_numpy(a).to(env.dev) for a in ids_np]
    cap = max(a.size for a in ids_np)
    out = torch.empty(cap * D, dtype=torch.float32, device=env.dev)
    sorted_dev = [torch.from_numpy(np.sort(a)).to(env.dev) for a in ids_np]
    kern_sorted = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, sorted_dev[:W] + sorted_dev, out, W)
    del sorted_dev
    kern = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev[:W] + ids_dev, out, W)
    ok = env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out)
    total_bytes = sum(a.size for a in ids_np) * D * 4
    # device-resident variant on a 16,000,000-row slice: IDs folded into the slice, de-duplicated again
    srows = 16_000_000
    devt = table.to_device(0, srows)
    folded = []
    for a in ids_np:
        f = a % srows
        _, first = np.unique(f, return_index=True)
        folded.append(np.ascontiguousarray(f[np.sort(first)]))
    fdev = [torch.from_numpy(a).to(env.dev) for a in folded]
    kern_h = _kernel_times(ud, torch, devt.device_ptr, srows, D, ud.UD_F32, fdev[:W] + fdev, out, W)
    ok_h = env.spot_check(table, srows, D, env.oracle.F32, folded[-1], out)
    hbm_bytes = sum(a.size for a in folded) * (2 * D * 4 + 8)
    devt.free()
    sizes = [a.size for a in ids_np]
    if not inputs:
        table.free()
    stated = N == LARGE_ROWS[0]
    return {"value": total_bytes / sum(kern) / 1e6, "ms_per_step": sum(kern) / nb, "dtype": "f32",
            "config": {"workload": f"large host-resident table: {N:,} x 256 fp32 ({N * D * 4 / 1e9:.1f} GB pinned"
                                   + ("" if stated else f"; the configuration's {LARGE_ROWS[0]:,} rows were refused by the host, see "
                                                        "table_allocation_attempts") +
                                   "), procedural Zipf graph, 1,024 seeds, fanout [15,10,5], de-duplicated; one step = one batch",
                       "unique_ids_per_batch": [min(sizes), max(sizes)], "table_rows": N, "stated_size": stated},
            "table_allocation_attempts": attempts, "table_ready_s": round(ready, 1),
            "kernel_only": _stats(kern), "rows_per_s": round(sum(sizes) / sum(kern) * 1e3),
            "sorted_ids_GBps": round(total_bytes / sum(kern_sorted) / 1e6, 2),
            "device_resident_slice": {"rows": srows, "GBps_read_plus_write": round(hbm_bytes / sum(kern_h) / 1e6, 1),
                                      "frac_of_8TBps": round(hbm_bytes / sum(kern_h) / 1e6 / HBM_PEAK_GBPS, 4),
                                      "kernel_only": _stats(kern_h), "parity_spot_check": ok_h},
            "parity_spot_check": ok and ok_h}


def wl_hybrid_case(env, name, table, N, ids_np, seed, fracs):
    """Hot-row cache in HBM over a host table: the most popular rows are read from HBM, the rest over the link."""
    ud, torch, np, workloads = env.ud, env.torch, env.np, env.workloads
    W, D = env.W, table.D
    stream = torch.cuda.current_stream().cuda_stream
    ids_dev = [torch.from_numpy(a).to(env.dev) for a in ids_np]
    out = torch.empty(max(a.size for a in ids_np) * D, dtype=torch.float32, device=env.dev)
    useful = sum(a.size for a in ids_np) * D * 4
    plain = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev[:W] + ids_dev, out, W)
    r = {"plain_zero_copy_GBps": round(useful / sum(plain) / 1e6, 2), "caches": {}}
    ok, last = True, None
    for frac in fracs:
        n_hot = int(N * frac)
        hot = workloads.hottest_nodes(N, n_hot, seed)
        cache = ud.Cache(table, hot)
        hits = int(np.isin(ids_np[0], hot).sum()) if n_hot <= 5_000_000 else -1
        seq = ids_dev[:W] + ids_dev
        ms = env.event_times(lambda k: ud.ud_gather_cached(cache.handle, ud.UD_F32, seq[k].data_ptr(), ud.UD_I64, seq[k].numel(),
                                                           out.data_ptr(), stream), len(seq), W)
        ok = ok and env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out)
        r["caches"][f"{frac:g}"] = {"rows_cached": n_hot, "hbm_GB": round(n_hot * D * 4 / 1e9 + N * 4 / 1e9, 2),
                                    "effective_GBps": round(useful / sum(ms) / 1e6, 2),
                                    "speedup_vs_plain": round(sum(plain) / sum(ms), 3),
                                    "hit_fraction_batch0": round(hits / ids_np[0].size, 4) if hits >= 0 else None,
                                    "kernel_only": _stats(ms)}
        last = (useful, sum(ms))
        cache.free()
    r["parity_spot_check"] = ok
    return r, last


def wl_hybrid(env, quick=False, products=None, papers=None):
    workloads = env.workloads
    nb = 5 if quick else 10
    cases, ok = {}, True
    tot_b = tot_ms = 0.0
    for name, given, maker, seed, fracs in (("products_like", products, _products_like_inputs, 3, (0.05, 0.2) if quick else (0.01, 0.05, 0.2)),
                                            ("papers_like", papers, _papers_like_inputs, 4, (0.05, 0.256) if quick else (0.01, 0.05, 0.256))):
        if given:
            table, N, ids_np = given
        else:
            made = maker(env, nb)
            table, N, ids_np = (made[0], made[0].N, made[1]) if name == "products_like" else (made[0], made[1], made[2])
        if table is None:
            continue
        r, last = wl_hybrid_case(env, name, table, N, ids_np[:nb], seed, fracs)
        cases[name] = r
        ok = ok and r["parity_spot_check"]
        tot_b += last[0]
        tot_ms += last[1]
        if not given:
            table.free()
    return {"value": tot_b / tot_ms / 1e6 if tot_ms else 0.0, "ms_per_step": tot_ms / (2 * nb), "dtype": "f32",
            "config": {"workload": "hybrid placement: hot-row cache in HBM (most popular rows by rank) over the host-pinned "
                                   "table, on the two GraphSAGE-style workloads; value = useful bytes / time with the "
                                   "largest cache; one step = one batch"},
            "cases": cases, "parity_spot_check": ok}


def wl_scatter(env, quick=False, table=None):
    """Write direction: rows scattered from HBM into the host-pinned table (distinct IDs)."""
    ud, torch, np, workloads, bl = env.ud, env.torch, env.np, env.workloads, env.bl
    W = env.W
    best, med = ctypes.c_double(), ctypes.c_double()
    bl.udb_d2h_peak(1 << 30, 10, ctypes.byref(best), ctypes.byref(med))
    d2h_peak = best.value
    N, M = N_ROWS, M_ROWS
    dmax = max(WIDTHS)
    own = table is None
    if own:
        table = ud.Table(N, dmax, ud.UD_F32)
        workloads.fill_uniform_f32(table.host_ptr, 8, N * dmax)
    src = torch.empty(M * dmax, dtype=torch.float32, device=env.dev).uniform_(-1, 1)
    reps = 4 if quick else min(env.K, 10)
    perms = [np.random.default_rng(k).permutation(N)[:M].astype(np.int64) for k in range(reps + W)]
    ids_dev = [torch.from_numpy(a).to(env.dev) for a in perms]
    stream = torch.cuda.current_stream().cuda_stream
    devt = table.to_device()
    rows, ok = {}, True
    tot_b = tot_ms = 0.0
    for D in WIDTHS:
        per = {}
        for where, tptr in (("host", table.device_ptr), ("hbm", devt.device_ptr)):
            ms = env.event_times(lambda k: ud.ud_scatter(tptr, N, D, ud.UD_F32, ids_dev[k].data_ptr(), ud.UD_I64, M, src.data_ptr(),
                                                         stream), len(ids_dev), W)
            per[where] = _stats(ms)
        # spot check on the host table: sampled rows of the last scatter equal their source rows
        samp = np.sort(np.random.default_rng(1).choice(M, 2048, replace=False))
        last = perms[-1]
        want = src[: M * D].view(M, D)[torch.from_numpy(samp).to(env.dev)].cpu().numpy()
        got = np.empty((samp.size, D), dtype=np.uint32)
        env.oracle.gather_raw(table.host_ptr, N, D, env.oracle.F32, np.ascontiguousarray(last[samp]), got)
        ok = ok and bool(np.array_equal(got, want.view(np.uint32)))
        nbytes = M * D * 4
        rows[str(D)] = {"row_bytes": D * 4, "host_ms": per["host"]["median_ms"],
                        "host_GBps": round(nbytes / per["host"]["median_ms"] / 1e6, 2),
                        "frac_of_d2h_peak": round(nbytes / per["host"]["median_ms"] / 1e6 / d2h_peak, 4),
                        "hbm_GBps_read_plus_write": round(2 * nbytes / per["hbm"]["median_ms"] / 1e6, 1)}
        tot_b += nbytes
        tot_ms += per["host"]["median_ms"]
    devt.free()
    if own:
        table.free()
    return {"value": tot_b / tot_ms / 1e6, "ms_per_step": tot_ms, "dtype": "f32",
            "config": {"workload": "write direction: 1,000,000 distinct rows scattered from HBM into a host-pinned fp32 table "
                                   "4,000,000 x D, D in {16,64,100,128,256,602}; one step = one scatter per width"},
            "d2h_peak_GBps": round(d2h_peak, 2), "per_width": rows, "frac_of_d2h_peak": round(tot_b / tot_ms / 1e6 / d2h_peak, 4),
            "parity_spot_check": ok}


def wl_overlap(env, quick=False, table=None):
    """Gather for batch b+1 on a second stream while a stand-in consumer works on batch b: how much of the
    gather time disappears behind compute."""
    ud, torch, np, workloads = env.ud, env.torch, env.np, env.workloads
    p = workloads.PAPERS_LIKE
    N, D = 16_000_000, p["D"]
    own = table is None
    if own:
        table = ud.Table(N, D, ud.UD_F32)
        workloads.fill_uniform_f32(table.host_ptr, 4, N * D)
    nb = 8 if quick else 12
    ids_np = [workloads.sample_procedural(N, p["degree"], p["alpha"], 4, p["nseeds"], p["fanout"], 44, b) for b in range(nb)]
    M = min(a.size for a in ids_np)
    ids_dev = [torch.from_numpy(np.ascontiguousarray(a[:M])).to(env.dev) for a in ids_np]
    bufs = [torch.empty((M, D), dtype=torch.float32, device=env.dev) for _ in range(2)]
    hidden = 1024
    w1 = torch.randn(D, hidden, device=env.dev) * 0.05
    w2 = torch.randn(hidden, hidden, device=env.dev) * 0.05
    layers = 1
    consumer = {"kind": "gemm"}
    scratch = torch.empty((M, D), dtype=torch.float32, device=env.dev)

    def consume(x):
        if consumer["kind"] == "gemm":                      # dense layers: MFMA-bound, statically partitioned kernels
            h = torch.relu(x @ w1)
            for _ in range(layers):
                h = torch.relu(h @ w2)
            return h.sum()
        for _ in range(consumer["passes"]):                 # element-wise passes: HBM-bound, many small workgroups
            torch.mul(x, 1.0001, out=scratch)
        return scratch

    sg, sc = torch.cuda.Stream(), torch.cuda.Stream()

    def gather_on(stream, b, buf, tun):
        ud.ud_gather_tuned(table.device_ptr, N, D, ud.UD_F32, ids_dev[b].data_ptr(), ud.UD_I64, M, buf.data_ptr(),
                           stream.cuda_stream, tun)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(2):                                   # the better of two: co-scheduling of two streams is jittery
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3
            best = ms if best is None or ms < best else best
        return best

    def only_gather(tun):
        def f():
            for b in range(nb):
                gather_on(sg, b, bufs[b & 1], tun)
        return f

    def only_compute():
        with torch.cuda.stream(sc):
            for b in range(nb):
                consume(bufs[b & 1])

    # size the consumer so that it takes a little longer than one gather
    t_g = timed(only_gather(None)) / nb
    while True:
        t_c = timed(only_compute) / nb
        if t_c >= 1.2 * t_g or layers >= 64:
            break
        layers = max(layers + 1, int(layers * 1.2 * t_g / max(t_c, 1e-3)))

    def serial(tun):
        def f():
            with torch.cuda.stream(sc):
                for b in range(nb):
                    gather_on(sc, b, bufs[b & 1], tun)
                    consume(bufs[b & 1])
        return f

    spans = {}

    def overlapped(tun):
        def f():
            g_start = [torch.cuda.Event(enable_timing=True) for _ in range(nb)]
            g_done = [torch.cuda.Event(enable_timing=True) for _ in range(nb)]
            c_start = [torch.cuda.Event(enable_timing=True) for _ in range(nb)]
            c_done = [torch.cuda.Event(enable_timing=True) for _ in range(nb)]
            for b in range(nb):
                if b >= 2:
                    sg.wait_event(c_done[b - 2])            # buffer b&1 is free again
                g_start[b].record(sg)
                gather_on(sg, b, bufs[b & 1], tun)
                g_done[b].record(sg)
                sc.wait_event(g_done[b])
                c_start[b].record(sc)
                with torch.cuda.stream(sc):
                    consume(bufs[b & 1])
                c_done[b].record(sc)
            torch.cuda.synchronize()
            mid = range(2, nb - 1)                          # steady state
            spans["gather"] = sum(g_start[b].elapsed_time(g_done[b]) for b in mid) / len(mid)
            spans["compute"] = sum(c_start[b].elapsed_time(c_done[b]) for b in mid) / len(mid)
        return f

    T = ud.ud_tuning
    shapes = [("auto", None), ("512wg_1row", T(0, 0, 1, 512, 0)), ("128wg_1row", T(0, 0, 1, 128, 0)), ("64wg_1row", T(0, 0, 1, 64, 0)),
              ("share_gpu_flag", T(0, 0, 0, 0, ud.UD_TUNE_SHARE_GPU))]
    if not quick:
        shapes += [("256wg", T(0, 0, 0, 256, 0)), ("64wg_4rows_in_flight", T(0, 1, 4, 64, 0)),
                   ("32wg_4rows_in_flight", T(0, 1, 4, 32, 0))]
    variants = {}
    for name, tun in shapes:
        tg = timed(only_gather(tun)) / nb
        ts = timed(serial(tun)) / nb
        to = timed(overlapped(tun)) / nb
        variants[name] = {"gather_only_ms": round(tg, 3), "serial_ms": round(ts, 3), "overlapped_ms": round(to, 3),
                          "gather_ms_while_overlapped": round(spans["gather"], 3),
                          "compute_ms_while_overlapped": round(spans["compute"], 3),
                          "exposed_gather_ms": round(max(to - t_c, 0.0), 3),
                          "hidden_fraction_of_gather": round(1.0 - max(to - t_c, 0.0) / tg, 3)}
    # the same pipeline with a bandwidth-bound, finely divided consumer of about the same length
    consumer.update(kind="elementwise", passes=8)
    t_e = timed(only_compute) / nb
    consumer["passes"] = max(1, round(8 * t_c / t_e))
    t_e = timed(only_compute) / nb
    elementwise = {"compute_only_ms": round(t_e, 3), "passes": consumer["passes"]}
    for name, tun in (("auto", None), ("512wg_1row", T(0, 0, 1, 512, 0)), ("128wg_1row", T(0, 0, 1, 128, 0)),
                      ("64wg_1row", T(0, 0, 1, 64, 0)), ("share_gpu_flag", T(0, 0, 0, 0, ud.UD_TUNE_SHARE_GPU))):
        tg = timed(only_gather(tun)) / nb
        to = timed(overlapped(tun)) / nb
        elementwise[name] = {"gather_only_ms": round(tg, 3), "overlapped_ms": round(to, 3),
                             "gather_ms_while_overlapped": round(spans["gather"], 3),
                             "compute_ms_while_overlapped": round(spans["compute"], 3),
                             "hidden_fraction_of_gather": round(1.0 - max(to - t_e, 0.0) / tg, 3)}
    consumer["kind"] = "gemm"
    ud.ud_gather_status(sg.cuda_stream)
    ud.ud_gather_status(sc.cuda_stream)
    ok = env.spot_check(table, N, D, env.oracle.F32, np.ascontiguousarray(ids_np[nb - 1][:M]), bufs[(nb - 1) & 1].view(-1))
    best = min(variants.values(), key=lambda v: v["overlapped_ms"])
    if own:
        table.free()
    return {"value": M * D * 4 / best["overlapped_ms"] / 1e6, "ms_per_step": best["overlapped_ms"], "dtype": "f32",
            "config": {"workload": f"overlap: zero-copy gather of batch b+1 ({M} rows x 1024 B from the first 16,000,000 rows of a host "
                                   f"table) on one stream while {layers + 1} dense fp32 layers (hidden {hidden}) consume batch b on "
                                   "another; value = gathered bytes / per-batch time of the overlapped pipeline"},
            "compute_only_ms": round(t_c, 3), "variants": variants, "elementwise_consumer": elementwise, "parity_spot_check": ok}


def wl_padded(env, quick=False, dense_table=None):
    """The same gathers from tables whose row pitch is rounded up to 128 bytes (UD_TABLE_PAD_ROWS): no row shares
    a memory line with its neighbours, so nothing but the row's own lines is fetched.  quick: the D=602 fp32 case
    only, its dense side being the table given."""
    ud, torch, np, workloads = env.ud, env.torch, env.np, env.workloads
    oracle = env.oracle
    N, M, W = N_ROWS, M_ROWS, env.W
    stream = torch.cuda.current_stream().cuda_stream
    reps = 4 if quick else min(env.K, 10)
    cases, ok = {}, True
    tot_b = tot_ms = 0.0
    todo = (("f32_D100", ud.UD_F32, ud.UD_F32, oracle.F32, 100), ("f32_D602", ud.UD_F32, ud.UD_F32, oracle.F32, 602),
            ("f16_to_f32_D602", ud.UD_F16, ud.UD_F16_TO_F32, oracle.F16_TO_F32, 602))
    if quick:
        todo = todo[1:2]
    for name, elem, dtype, odtype, D in todo:
        esz = 4 if elem == ud.UD_F32 else 2
        ids_np = [workloads.indices_uniform(workloads.IDX_STREAM + k, M, N) for k in range(reps + W)]
        ids_dev = [torch.from_numpy(a).to(env.dev) for a in ids_np]
        out = torch.empty(M * D, dtype=torch.float32, device=env.dev)
        r = {}
        for kind, flags in (("dense", 0), ("padded", ud.UD_TABLE_PAD_ROWS)):
            given = kind == "dense" and dense_table is not None and dense_table.D == D and dense_table.elem == elem
            t = dense_table if given else ud.Table(N, D, elem, flags)
            if not given:
                (workloads.fill_uniform_f32 if elem == ud.UD_F32 else workloads.fill_normal_f16)(t.host_ptr, 9, N * t.pitch)
            ms = env.event_times(lambda k: ud.ud_gather_pitched(t.device_ptr, N, D, t.pitch, dtype, ids_dev[k].data_ptr(), ud.UD_I64, M,
                                                                out.data_ptr(), stream), len(ids_dev), W)
            st = _stats(ms)
            ok = ok and env.spot_check(t, N, D, odtype, ids_np[-1], out, pitch=t.pitch)
            useful = M * D * esz
            r[kind] = {"pitch_bytes": t.pitch * esz, "ms": st["median_ms"], "GBps": round(useful / st["median_ms"] / 1e6, 2),
                       "frac_of_h2d_peak": round(useful / st["median_ms"] / 1e6 / env.h2d_peak, 4),
                       "table_GB": round(t.nbytes / 1e9, 2)}
            if kind == "padded":
                tot_b += useful
                tot_ms += st["median_ms"]
            if not given:
                t.free()
        r["speedup"] = round(r["dense"]["ms"] / r["padded"]["ms"], 3)
        cases[name] = r
    return {"value": tot_b / tot_ms / 1e6, "ms_per_step": tot_ms, "dtype": "f32",
            "config": {"workload": "padded rows: 1,000,000 int64 IDs from 4,000,000-row host-pinned tables with the row pitch "
                                   "rounded up to 128 bytes, against the dense layout; value = useful bytes / time, padded tables"},
            "padded_cases": cases, "parity_spot_check": ok}


def wl_fp16(env, quick=False):
    ud, torch, np, workloads = env.ud, env.torch, env.np, env.workloads
    W = env.W
    N, D, M = 10_000_000, 602, 2_000_000
    t0 = time.perf_counter()
    table = ud.Table(N, D, ud.UD_F16)
    workloads.fill_normal_f16(table.host_ptr, 5, N * D)
    ready = time.perf_counter() - t0
    reps = 5 if quick else min(env.K, 10)
    ids_np = [workloads.indices_uniform(workloads.IDX_STREAM + k, M, N, np.int32) for k in range(reps + W)]
    ids_dev = [torch.from_numpy(a).to(env.dev) for a in ids_np]
    out = torch.empty(M * D, dtype=torch.float32, device=env.dev)
    kern = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F16_TO_F32, ids_dev, out, W)
    ok = env.spot_check(table, N, D, env.oracle.F16_TO_F32, ids_np[-1], out)
    wall = _wall_times(ud, torch, table.device_ptr, N, D, ud.UD_F16_TO_F32, [env.pinned(a) for a in ids_np], out, W)
    table.free()
    ks = _stats(kern)
    link_bytes = M * D * 2
    return {"value": link_bytes / ks["median_ms"] / 1e6, "ms_per_step": ks["median_ms"], "dtype": "f16->f32",
            "config": {"workload": "half-precision odd-width table: host-pinned fp16 10,000,000 x 602 (N(0,1) rounded to fp16), "
                                   "2,000,000 int32 IDs uniform, fused upcast to fp32 in HBM"},
            "kernel_only": ks, "call_to_sync_incl_id_copy": _stats(wall), "table_ready_s": round(ready, 1),
            "hbm_write_GBps": round(2 * link_bytes / ks["median_ms"] / 1e6, 2),
            # a dense table of 1204-byte rows overlaps 10.375 128-byte lines per row on average
            "line_floor_frac_of_h2d_peak": round(1204 / (10.375 * 128), 4),
            "rows_per_s": round(M / ks["median_ms"] * 1e3), "parity_spot_check": ok}


def wl_align(env, quick=False, table=None):
    """Section 5.3 / Figure 7 of the paper: row sizes 2048..2076 bytes in 4-byte steps."""
    ud, torch, np, workloads, bl = env.ud, env.torch, env.np, env.workloads, env.bl
    W, threads = env.W, env.threads
    N, M = 4_000_000, 262_144
    widths = list(range(512, 520))
    dmax = widths[-1]
    own = table is None
    if own:
        table = ud.Table(N, dmax, ud.UD_F32)
        workloads.fill_uniform_f32(table.host_ptr, 7, N * dmax)
    assert table.N * table.D >= N * dmax
    reps = 4 if quick else max(env.K, 5)
    ids_np = [workloads.indices_uniform(workloads.IDX_STREAM + k, M, N) for k in range(reps + W)]
    ids_dev = [torch.from_numpy(a).to(env.dev) for a in ids_np]
    out = torch.empty(M * dmax, dtype=torch.float32, device=env.dev)
    ctx = ctypes.c_void_p()
    have_cpu = not env.no_cpu and bl.udb_cpu_centric_create(M * dmax * 4, ctypes.byref(ctx)) == 0
    naive = ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_ELEMENTWISE)
    shifted = ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_ELEMENTWISE | ud.UD_TUNE_CIRCULAR_SHIFT)
    rows, ok = {}, True
    for D in widths:
        nbytes = M * D * 4
        opt = _stats(_kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W))
        ok = ok and env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out)
        nv = _stats(_kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W, naive))
        ok = ok and env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out, 256)
        sh = _stats(_kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W, shifted))
        ok = ok and env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out, 256)
        r = {"zero_copy_ms": opt["median_ms"], "zero_copy_GBps": round(nbytes / opt["median_ms"] / 1e6, 2),
             "one_lane_per_element_ms": nv["median_ms"], "one_lane_per_element_GBps": round(nbytes / nv["median_ms"] / 1e6, 2),
             "circular_shift_ms": sh["median_ms"], "circular_shift_GBps": round(nbytes / sh["median_ms"] / 1e6, 2),
             "ideal_ms": round(nbytes / env.h2d_peak / 1e6, 4)}
        if have_cpu:
            _cpu_centric(bl, ctx, table.host_ptr, D * 4, ids_np[0], out.data_ptr(), threads)
            cpu = sorted(_cpu_centric(bl, ctx, table.host_ptr, D * 4, a, out.data_ptr(), threads) for a in ids_np[1:4 if quick else 6])
            py = cpu[len(cpu) // 2]
            r.update({"cpu_centric_ms": round(py, 4), "speedup_vs_cpu_centric": round(py / opt["median_ms"], 3),
                      "one_lane_per_element_speedup_vs_cpu_centric": round(py / nv["median_ms"], 3)})
        rows[str(D * 4)] = r
    if have_cpu:
        bl.udb_cpu_centric_destroy(ctx)
    if own:
        table.free()
    tot_b = sum(M * D * 4 for D in widths)
    tot_ms = sum(r["zero_copy_ms"] for r in rows.values())
    return {"value": tot_b / tot_ms / 1e6, "ms_per_step": tot_ms, "dtype": "f32",
            "config": {"workload": "alignment sweep: host-pinned fp32 table 4,000,000 rows, row bytes 2048..2076 step 4, "
                                   "262,144 int64 IDs uniform; one step = one gather per row size", "cpu_centric_threads": threads},
            "per_row_bytes": rows, "parity_spot_check": ok}


def wl_grid(env, quick=False):
    """Section 5.2 / Figure 6 of the paper: (rows copied, row bytes) from (8K, 256B) to (256K, 16KB)."""
    ud, torch, np, workloads, bl = env.ud, env.torch, env.np, env.workloads, env.bl
    W, threads = env.W, env.threads
    region = 16 << 30
    table = ud.Table(region // 16384, 4096, ud.UD_F32)      # 16 GiB, viewed with each row size
    workloads.fill_uniform_f32(table.host_ptr, 6, region // 4)
    reps = 3 if quick else max(env.K, 5)
    ctx = ctypes.c_void_p()
    have_cpu = not env.no_cpu and bl.udb_cpu_centric_create(262_144 * 16384, ctypes.byref(ctx)) == 0
    out = torch.empty(262_144 * 4096, dtype=torch.float32, device=env.dev)
    naive = ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_ELEMENTWISE)
    cells, ok = {}, True
    tot_b = tot_ms = 0.0
    for rb in (256, 1024, 4096, 16384):
        D, N = rb // 4, region // rb
        for M in (8_192, 32_768, 131_072, 262_144):
            ids_np = [workloads.indices_uniform(workloads.IDX_STREAM + k, M, N) for k in range(reps + W)]
            ids_dev = [torch.from_numpy(a).to(env.dev) for a in ids_np]
            nbytes = M * rb
            kern = _stats(_kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W))
            ok = ok and env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out, 512)
            nv = _stats(_kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W, naive))
            ok = ok and env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out, 128)
            pinned = [env.pinned(a) for a in ids_np]
            wall = _stats(_wall_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, pinned, out, W))
            wall_zc = _stats(_wall_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, pinned, out, W, ids_stay_in_host=True))
            ok = ok and env.spot_check(table, N, D, env.oracle.F32, ids_np[-1], out, 128)
            ideal = nbytes / env.h2d_peak / 1e6
            c = {"MB": round(nbytes / 1e6, 2), "kernel_ms": kern["median_ms"], "one_lane_per_element_kernel_ms": nv["median_ms"],
                 "call_to_sync_ms": wall["median_ms"], "ideal_ms": round(ideal, 4),
                 "slowdown_vs_ideal": round(wall["median_ms"] / ideal, 3),
                 "call_to_sync_ids_read_from_host_ms": wall_zc["median_ms"],
                 "ids_read_from_host_slowdown_vs_ideal": round(wall_zc["median_ms"] / ideal, 3),
                 "one_lane_per_element_kernel_slowdown_vs_ideal": round(nv["median_ms"] / ideal, 3)}
            if have_cpu:
                _cpu_centric(bl, ctx, table.host_ptr, rb, ids_np[0], out.data_ptr(), threads)
                cpu = sorted(_cpu_centric(bl, ctx, table.host_ptr, rb, a, out.data_ptr(), threads) for a in ids_np[1:1 + min(reps, 5)])
                py = cpu[len(cpu) // 2]
                c.update({"cpu_centric_ms": round(py, 4), "cpu_centric_slowdown_vs_ideal": round(py / ideal, 3),
                          "speedup_vs_cpu_centric": round(py / wall["median_ms"], 3)})
            cells[f"({M // 1024}K, {rb}B)"] = c
            tot_b += nbytes
            tot_ms += kern["median_ms"]
    if have_cpu:
        bl.udb_cpu_centric_destroy(ctx)
    table.free()
    return {"value": tot_b / tot_ms / 1e6, "ms_per_step": tot_ms, "dtype": "f32",
            "config": {"workload": "size grid: 16 GiB host-pinned fp32 region viewed as rows of 256 B..16 KB, "
                                   "8K..256K int64 IDs uniform; call-to-sync times include the ID list's H2D copy; "
                                   "one step = one gather per cell", "cpu_centric_threads": threads},
            "cells": cells, "parity_spot_check": ok}


WORKLOADS = {"single": wl_single, "graphsage": wl_graphsage, "large": wl_large, "fp16": wl_fp16, "align": wl_align, "grid": wl_grid,
             "hybrid": wl_hybrid, "scatter": wl_scatter, "overlap": wl_overlap, "padded": wl_padded}


def _round_floats(x, nd=3):
    if isinstance(x, float):
        return round(x, nd)
    if isinstance(x, dict):
        return {k: _round_floats(v, nd) for k, v in x.items()}
    if isinstance(x, list):
        return [_round_floats(v, nd) for v in x]
    return x


def _embed(env, res):
    """A workload's result boiled down for the all-in-one line (the line has to stay well below what the harness
    keeps of stdout); the full dictionaries go to gpurun_out/bench_details.json."""
    out = {"GBps": round(res["value"], 2), "frac_of_h2d_peak": round(res["value"] / env.h2d_peak, 4),
           "ms_per_step": round(res["ms_per_step"], 4), "dtype": res["dtype"], "parity_spot_check": res.get("parity_spot_check")}
    if "kernel_only" in res:
        out["kernel_ms"] = res["kernel_only"]["median_ms"]
    if "call_to_sync_incl_id_copy" in res:
        out["call_to_sync_ms_incl_id_copy"] = res["call_to_sync_incl_id_copy"]["median_ms"]
    for k in ("frac_of_same_size_hipMemcpy", "sorted_ids_GBps", "rows_per_s", "hbm_write_GBps", "line_floor_frac_of_h2d_peak",
              "table_allocation_attempts", "d2h_peak_GBps", "frac_of_d2h_peak", "compute_only_ms"):
        if k in res:
            out[k] = res[k]
    if "hip_graph_replay_call_to_sync" in res:
        out["hip_graph_replay_call_to_sync_ms"] = res["hip_graph_replay_call_to_sync"]["median_ms"]
    cfg = res.get("config", {})
    for k in ("unique_ids_per_batch", "batches", "table_rows", "stated_size"):
        if k in cfg:
            out[k] = cfg[k]
    if res.get("cpu_centric"):
        out["cpu_centric_GBps"] = {k: v["GBps"] for k, v in res["cpu_centric"].items()}
    if "device_resident_slice" in res:
        d = res["device_resident_slice"]
        out["hbm_slice"] = {"rows": d["rows"], "GBps_read_plus_write": d["GBps_read_plus_write"], "frac_of_8TBps": d["frac_of_8TBps"],
                            "kernel_ms": d["kernel_only"]["median_ms"], "parity_spot_check": d["parity_spot_check"]}
    if "per_row_bytes" in res:          # alignment sweep
        out["columns"] = ["zero_copy_GBps", "one_lane_per_element_GBps", "circular_shift_GBps", "cpu_centric_ms", "zero_copy_ms", "ideal_ms"]
        out["per_row_bytes"] = {k: [v["zero_copy_GBps"], v["one_lane_per_element_GBps"], v["circular_shift_GBps"],
                                    v.get("cpu_centric_ms"), v["zero_copy_ms"], v["ideal_ms"]] for k, v in res["per_row_bytes"].items()}
    if "cells" in res:                  # size grid
        out["columns"] = ["MB", "call_to_sync_x_ideal", "one_lane_per_element_kernel_x_ideal", "cpu_centric_x_ideal", "call_to_sync_ms",
                          "call_to_sync_ids_read_from_host_x_ideal"]
        out["cells"] = {k: [v["MB"], v["slowdown_vs_ideal"], v["one_lane_per_element_kernel_slowdown_vs_ideal"],
                            v.get("cpu_centric_slowdown_vs_ideal"), v["call_to_sync_ms"], v["ids_read_from_host_slowdown_vs_ideal"]]
                        for k, v in res["cells"].items()}
    if "per_width" in res:              # write direction
        out["columns"] = ["host_GBps", "frac_of_d2h_peak", "hbm_GBps_read_plus_write"]
        out["per_width"] = {k: [v["host_GBps"], v["frac_of_d2h_peak"], v["hbm_GBps_read_plus_write"]] for k, v in res["per_width"].items()}
    if "cases" in res and "config" in res and "hybrid" in res["config"]["workload"]:
        out["columns"] = ["rows_cached", "hit_fraction_batch0", "effective_GBps", "speedup_vs_plain"]
        out["cases"] = {name: {"plain_zero_copy_GBps": c["plain_zero_copy_GBps"],
                               "caches": {f: [v["rows_cached"], v["hit_fraction_batch0"], v["effective_GBps"], v["speedup_vs_plain"]]
                                          for f, v in c["caches"].items()}} for name, c in res["cases"].items()}
    if "padded_cases" in res:           # 128-byte row pitch against the dense layout
        out["columns"] = ["pitch_bytes", "GBps", "frac_of_h2d_peak"]
        out["cases"] = {name: {k: ([v["pitch_bytes"], v["GBps"], v["frac_of_h2d_peak"]] if isinstance(v, dict) else v)
                               for k, v in c.items()} for name, c in res["padded_cases"].items()}
    if "variants" in res:               # overlap with a consumer
        out["columns"] = ["gather_only_ms", "overlapped_ms", "hidden_fraction_of_gather"]
        out["gemm_consumer"] = {k: [v["gather_only_ms"], v["overlapped_ms"], v["hidden_fraction_of_gather"]] for k, v in res["variants"].items()}
        ec = res["elementwise_consumer"]
        out["elementwise_consumer"] = {"compute_only_ms": ec["compute_only_ms"],
                                       **{k: [v["gather_only_ms"], v["overlapped_ms"], v["hidden_fraction_of_gather"]]
                                          for k, v in ec.items() if isinstance(v, dict)}}
    return _round_floats(out, 4)


def run_one(env, name) -> int:
    """One of the other configurations / experiments as a bench line of its own."""
    torch = env.torch
    res = WORKLOADS[name](env)
    line = {"metric": "zero_copy_gather_GBps", "value": round(res["value"], 3), "unit": "GB/s", "n_gpus": 1, "steps": env.K,
            "warmup": env.W, "ms_per_step": round(res["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": res["dtype"], "data": "synthetic", "config": res["config"],
            "h2d_peak_GBps": round(env.h2d_peak, 2), "frac_of_h2d_peak": round(res["value"] / env.h2d_peak, 4),
            "host": {"cores_visible": env.ncores, "device": torch.cuda.get_device_name(0)}, "build_id": env.ud.ud_build_id()}
    for k, v in res.items():
        if k not in ("value", "ms_per_step", "dtype", "config"):
            line[k] = _round_floats(v, 4)
    print(json.dumps(line))
    return 0 if res.get("parity_spot_check", True) else 1


def run_everything_else(env, sweep_table):
    """After the headline: every other configuration and experiment, few repetitions each, into two objects of the
    same line.  Pinned memory is limited (about 65 GiB on the development boxes), so tables are made and freed in
    turn; the sweep's own table serves the alignment sweep and, last, the write direction (which overwrites it)."""
    configs, experiments, timing, details = {}, {}, {}, {}

    def run(name, where, fn):
        t0 = time.perf_counter()
        try:
            res = fn()
            details[name] = _round_floats(res, 4)
            where[name] = _embed(env, res)
        except Exception as e:                       # one failing extra must not take the headline with it
            where[name] = {"error": f"{type(e).__name__}: {e}", "parity_spot_check": False}
        timing[name] = round(time.perf_counter() - t0, 1)
        env.torch.cuda.synchronize()

    run("align_fig7", experiments, lambda: wl_align(env, True, sweep_table))
    run("padded_rows", experiments, lambda: wl_padded(env, True, sweep_table))
    run("scatter", experiments, lambda: wl_scatter(env, True, sweep_table))
    sweep_table.free()
    run("config1_single", configs, lambda: wl_single(env, True))
    run("config5_fp16", configs, lambda: wl_fp16(env, True))
    prod = _products_like_inputs(env, 20)
    run("config3_graphsage", configs, lambda: wl_graphsage(env, True, prod))
    run("hybrid_products_like", experiments, lambda: wl_hybrid(env, True, products=(prod[0], prod[0].N, prod[1]), papers=(None, 0, [])))
    prod[0].free()
    del prod
    run("grid_fig6", experiments, lambda: wl_grid(env, True))
    pap = _papers_like_inputs(env, 5)
    run("config4_large", configs, lambda: wl_large(env, True, pap))
    if pap[0] is not None:
        run("hybrid_papers_like", experiments, lambda: wl_hybrid(env, True, products=(None, 0, []), papers=(pap[0], pap[1], pap[2])))
        run("overlap", experiments, lambda: wl_overlap(env, True, pap[0]))
        pap[0].free()
    try:                                             # the uncondensed results, where a harness collects output files
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "bench_details.json"), "w") as f:
            json.dump(details, f)
    except OSError:
        pass
    return configs, experiments, timing


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--threads", type=int, default=0, help="host threads of the CPU-centric baseline (0 = all)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the host baselines (for profiling runs)")
    ap.add_argument("--headline-only", action="store_true",
                    help="sweep workload: stop after the headline microbenchmark (no other configurations or experiments)")
    ap.add_argument("--workload", default="sweep",
                    choices=("sweep", "single", "graphsage", "large", "fp16", "align", "grid", "hybrid", "scatter", "overlap", "padded"),
                    help="sweep (default, the headline microbenchmark) or one of the other configurations / "
                         "the paper's alignment and size experiments")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the host-link gather has no multi-GPU path); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    from paper_2101_07956_amd import build as hip_build
    hip_build.ensure_built()            # builds only if no library is there or its stamp differs from the sources
    import paper_2101_07956_amd as ud
    import workloads

    bl = _load_baseline_lib(ud)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    K, W = args.steps, args.warmup
    ncores = len(os.sched_getaffinity(0))
    threads = args.threads or min(ncores, 16)
    t_start = time.perf_counter()
    # ---- host-link peak: best of 10 pinned hipMemcpy H2D of 1 GiB, same process (inside Env) ----
    env = Env(ud, bl, workloads, torch, np, threads, ncores, K, W, args.no_cpu)
    if args.workload != "sweep":
        return run_one(env, args.workload)
    h2d_peak = env.h2d_peak
    best, med = ctypes.c_double(), ctypes.c_double()
    bl.udb_d2d_peak(1 << 30, 10, ctypes.byref(best), ctypes.byref(med))
    d2d_copy = best.value

    # ---- inputs: one flat value stream, viewed as 4,000,000 x D for each width ----
    dmax = max(WIDTHS)
    table = ud.Table(N_ROWS, dmax, ud.UD_F32)
    workloads.fill_uniform_f32(table.host_ptr, TABLE_SEED, N_ROWS * dmax)
    ids_host = workloads.indices_uniform(workloads.IDX_STREAM, (K + W) * M_ROWS, N_ROWS).reshape(K + W, M_ROWS)
    ids = torch.from_numpy(ids_host).to(dev)
    out = torch.empty(M_ROWS * dmax, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    # a plain 1 GiB device copy of known size: the yardstick hardware byte counters are scaled by
    # when this command runs under rocprofv3 --pmc (2.4 GB of `out` is free to use as both ends)
    cal_bytes = 1 << 30
    bl.udb_plain_copy(out.data_ptr() + cal_bytes, out.data_ptr(), cal_bytes, stream)

    def step(s, tptr, events=None):
        for D in WIDTHS:
            if events is not None:
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
            ud.ud_gather(tptr, N_ROWS, D, ud.UD_F32, ids[s].data_ptr(), ud.UD_I64, M_ROWS, out.data_ptr(), stream)
            if events is not None:
                e1.record()
                events[D].append((e0, e1))

    def timed(tptr):
        for s in range(W):
            step(s, tptr)
        events = {D: [] for D in WIDTHS}
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(W, W + K):
            step(s, tptr, events)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        ud.ud_gather_status(stream)          # raises if any ID was out of range
        raw = {D: [a.elapsed_time(b) for a, b in ev] for D, ev in events.items()}
        per = {D: sum(v) / len(v) for D, v in raw.items()}                                       # mean ms per launch
        timed.spread = {D: (sorted(v)[len(v) // 2], min(v)) for D, v in raw.items()}             # median, min
        return elapsed, per

    elapsed, per_ms = timed(table.device_ptr)
    bytes_per_step = sum(M_ROWS * D * 4 for D in WIDTHS)
    value = K * bytes_per_step / elapsed / 1e9
    rows_per_s = K * M_ROWS * len(WIDTHS) / elapsed
    spread = dict(timed.spread)
    per_width = {
        str(D): {"row_bytes": D * 4, "ms": round(per_ms[D], 4), "ms_median": round(spread[D][0], 4),
                 "ms_min": round(spread[D][1], 4), "GBps": round(M_ROWS * D * 4 / per_ms[D] / 1e6, 2),
                 "frac_of_h2d_peak": round(M_ROWS * D * 4 / per_ms[D] / 1e6 / h2d_peak, 4),
                 "rows_per_s": round(M_ROWS / per_ms[D] * 1e3)}
        for D in WIDTHS
    }

    # ---- secondary timing: call to stream-sync per gather, including the ID list's host-to-device copy ----
    pinned_ids = [torch.from_numpy(ids_host[s]).pin_memory() for s in range(W + K)]
    wall = {}
    for D in WIDTHS:
        ms = _wall_times(ud, torch, table.device_ptr, N_ROWS, D, ud.UD_F32, pinned_ids, out, W)
        st = _stats(ms)
        wall[str(D)] = {"median_ms": st["median_ms"], "min_ms": st["min_ms"],
                        "GBps": round(M_ROWS * D * 4 / st["median_ms"] / 1e6, 2)}
    del pinned_ids
    step(W + K - 1, table.device_ptr)            # leave the last step's D=602 result in `out` for the spot check
    torch.cuda.synchronize()

    # ---- parity spot check of the last step's last gather against the oracle (outside the timed region) ----
    import oracle
    sample = np.random.default_rng(0).choice(M_ROWS, 4096, replace=False)
    sample.sort()
    last_ids = ids_host[W + K - 1]
    got = out[: M_ROWS * dmax].view(M_ROWS, dmax)[torch.from_numpy(sample).to(dev)].cpu().numpy()
    want = np.empty((sample.size, dmax), dtype=np.uint32)
    oracle.gather_raw(table.host_ptr, N_ROWS, dmax, oracle.F32, np.ascontiguousarray(last_ids[sample]), want)
    parity_ok = bool(np.array_equal(got.view(np.uint32), want))

    # ---- device-resident variant: same steps, table copied to HBM ----
    dev_table = table.to_device()
    elapsed_hbm, per_ms_hbm = timed(dev_table.device_ptr)
    hbm_traffic, hbm_traffic_note = _read_traffic_note(ud, dev_table.device_ptr, "hbm_variant_traffic_bytes_per_launch", "hbm_plan")
    hp = ud.ud_gather_plan(dev_table.device_ptr, 602, ud.UD_F32)
    hbm_kernel = ("gather_flat<f32> (destination-aligned)" if hp.flags & ud.UD_TUNE_DEST_ALIGNED else "gather_chunked<f32>") + \
        " D=602, table in HBM"
    dev_table.free()
    hbm_bytes_602 = M_ROWS * (2 * 602 * 4 + 8)       # row read + row write + one int64 ID
    hbm_achieved = hbm_bytes_602 / per_ms_hbm[602] / 1e6

    # ---- host baselines ----
    cpu_baseline = None
    cpu_centric = None
    if not args.no_cpu:
        # oracle, single thread, as it stands: whole steps (six widths x 1,000,000 rows each, a fresh ID
        # list per step) until at least 10 s of CPU work have been timed
        obuf = np.empty(M_ROWS * dmax, dtype=np.uint32)
        t_oracle, osteps = 0.0, 0
        while t_oracle < 10.0 and osteps < K + W:
            t0 = time.perf_counter()
            for D in WIDTHS:
                oracle.gather_raw(table.host_ptr, N_ROWS, D, oracle.F32, ids_host[osteps], obuf[: M_ROWS * D].reshape(M_ROWS, D))
            t_oracle += time.perf_counter() - t0
            osteps += 1
        cpu_baseline = {"value": round(osteps * bytes_per_step / t_oracle / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
                        "sample": f"{osteps} steps of the same workload (6 widths x 1,000,000 rows, {osteps * bytes_per_step / 1e9:.1f} GB gathered)",
                        "seconds": round(t_oracle, 2), "rows_per_s": round(osteps * M_ROWS * len(WIDTHS) / t_oracle)}
        del obuf
        # CPU-centric path: gather into pinned staging, then DMA (plain and double-buffered)
        ctx = ctypes.c_void_p()
        if bl.udb_cpu_centric_create(M_ROWS * dmax * 4, ctypes.byref(ctx)) == 0:
            res = {}
            a, b, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()

            def centric_step(s, th, slices):
                tot = [0.0, 0.0, 0.0]
                for D in WIDTHS:
                    rc = bl.udb_cpu_centric_gather(ctx, table.host_ptr, D * 4, ids_host[s].ctypes.data, M_ROWS,
                                                   out.data_ptr(), th, slices, ctypes.byref(a), ctypes.byref(b),
                                                   ctypes.byref(c))
                    if rc != 0:
                        raise RuntimeError(f"cpu-centric baseline failed ({rc})")
                    tot = [tot[0] + a.value, tot[1] + b.value, tot[2] + c.value]
                return tot

            for name, th, slices, reps in (("plain", threads, 1, 3), ("double_buffered", threads, 8, 3),
                                           ("plain_1thread", 1, 1, 1)):
                if th > 1:
                    centric_step(0, th, slices)                       # warm-up
                acc = [0.0, 0.0, 0.0]
                for rep in range(reps):
                    t = centric_step(1 + rep, th, slices)
                    acc = [acc[k] + t[k] for k in range(3)]
                res[name] = {"GBps": round(reps * bytes_per_step / acc[0] / 1e9, 2), "threads": th,
                             "gather_s_per_step": round(acc[1] / reps, 4),
                             "copy_s_per_step": round(acc[2] / reps, 4) if slices == 1 else None}
            bl.udb_cpu_centric_destroy(ctx)
            cpu_centric = res

    dom_ms = per_ms[602]
    dom_achieved = M_ROWS * 602 * 4 / dom_ms / 1e6
    traffic, traffic_note = _read_traffic_note(ud, table.device_ptr, "traffic_bytes_per_launch", "plan")
    # ---- every other configuration and experiment, few repetitions each (frees the table) ----
    configs = experiments = extras_seconds = None
    t_headline = time.perf_counter() - t_start
    if args.headline_only:
        table.free()
    else:
        try:
            configs, experiments, extras_seconds = run_everything_else(env, table)
        except Exception as e:                       # whatever escapes the per-entry handling: the headline still prints
            configs = experiments = {"all": {"error": f"{type(e).__name__}: {e}", "parity_spot_check": False}}
            extras_seconds = {}
    line = {
        "metric": "zero_copy_gather_GBps",
        "value": round(value, 3),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(elapsed / K * 1e3, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "gather microbenchmark sweep: host-pinned fp32 table 4,000,000 x D, "
                               "D in {16,64,100,128,256,602}, 1,000,000 int64 IDs uniform with replacement, seed 1; "
                               "one step = one gather per width",
                   "table": "pinned host memory (zero-copy)", "N": N_ROWS, "M": M_ROWS, "widths": list(WIDTHS)},
        "frac_of_h2d_peak": round(value / h2d_peak, 4),
        "min_frac_of_h2d_peak_rows_ge_512B": min(per_width[str(D)]["frac_of_h2d_peak"] for D in WIDTHS if D * 4 >= 512),
        "theoretical_link_GBps": 63.0,          # PCIe Gen5 x16 after 128b/130b encoding, before packet overhead: context only
        "rows_per_s": round(rows_per_s),
        "h2d_peak_GBps": round(h2d_peak, 2),
        "per_width": per_width,
        "call_to_sync_incl_id_copy": wall,
        "parity_spot_check": parity_ok,
        "roofline": {"bound": "host_link", "kernel": "gather_chunked<f32> D=602 (2408-byte rows)",
                     "achieved": round(dom_achieved, 2), "peak": round(h2d_peak, 2), "unit": "GB/s",
                     "frac": round(dom_achieved / h2d_peak, 4), "traffic": traffic, "traffic_note": traffic_note,
                     "traffic_unit": "bytes per launch (L2<->fabric reads + writes, rocprofv3 FETCH_SIZE/WRITE_SIZE)",
                     "algorithmic_bytes_per_launch": M_ROWS * (2 * 602 * 4 + 8),
                     "link_bytes_per_launch": M_ROWS * 602 * 4,
                     # a dense table of 2408-byte rows makes a row overlap 19.75 128-byte lines on average (the
                     # hardware fetches whole lines): the most a gather of this layout can show is 2408 / 2528 of the peak
                     "line_floor_bytes_per_launch": int(M_ROWS * 19.75 * 128),
                     "frac_incl_line_padding": round(M_ROWS * 19.75 * 128 / dom_ms / 1e6 / h2d_peak, 4),
                     "peak_source": "best of 10 pinned hipMemcpy H2D of 1 GiB in this run",
                     "ms_per_launch": round(dom_ms, 4)},
        "roofline_hbm": {"bound": "hbm", "kernel": hbm_kernel,
                         "achieved": round(hbm_achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": round(hbm_achieved / HBM_PEAK_GBPS, 4),
                         "traffic": hbm_traffic, "traffic_note": hbm_traffic_note,
                         "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE)",
                         "algorithmic_bytes_per_launch": hbm_bytes_602,
                         "per_width_GBps_read_plus_write": {str(D): round(M_ROWS * (2 * D * 4 + 8) / per_ms_hbm[D] / 1e6, 1)
                                                            for D in WIDTHS},
                         "ms_per_launch": round(per_ms_hbm[602], 4),
                         "sweep_GBps_read_plus_write": round(K * 2 * bytes_per_step / elapsed_hbm / 1e9, 1),
                         "d2d_memcpy_traffic_GBps": round(2 * d2d_copy, 1)},
        "cpu_baseline": cpu_baseline,
        "cpu_centric": cpu_centric,
        "configs": configs,
        "experiments": experiments,
        "seconds": {"headline": round(t_headline, 1), "extras": extras_seconds, "total": round(time.perf_counter() - t_start, 1)},
        "host": {"cores_visible": ncores, "device": torch.cuda.get_device_name(0), **_host_topology()},
        "build_id": ud.ud_build_id(),
    }
    print(json.dumps(line))
    extras_ok = all(v.get("parity_spot_check", True) for d in (configs, experiments) if d for v in d.values())
    return 0 if parity_ok and extras_ok else 1


if __name__ == "__main__":
    sys.exit(main())
