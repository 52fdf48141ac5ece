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
  roofline_hbm = the device-resident variant (same kernel, table in HBM) vs 8 TB/s
  cpu_baseline = the CPU oracle timed on this machine's host cores
  cpu_centric  = the path the paper argues against (CPU gather -> pinned staging
                 -> hipMemcpyAsync), plain and double-buffered
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


def _read_traffic_note(key="traffic_bytes_per_launch"):
    """Fabric traffic (bytes per launch) of the dominant kernel, measured offline with rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE and kept in the committed counter summary; None if that file is absent."""
    path = os.path.join(ROOT, "profiles", "gather_f32_D602_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith(key + "="):
            return float(line.split("=", 1)[1])
    return None


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


def _wall_times(ud, torch, tptr, N, D, dtype, ids_pinned, out, warm):
    """Call-to-sync wall time per gather INCLUDING the host->device copy of the ID list (pinned source)."""
    stream = torch.cuda.current_stream()
    dst = torch.empty(max(t.numel() for t in ids_pinned), dtype=ids_pinned[0].dtype, device="cuda")
    ms = []
    for k, ids in enumerate(ids_pinned):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        d = dst[: ids.numel()]
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


def run_other(args, ud, bl, workloads, torch, np, threads, ncores) -> int:
    """The other configurations and the paper's two microbenchmark experiments (not the default bench line)."""
    import oracle

    K, W = args.steps, args.warmup
    h2d_peak = _h2d_rate(bl, 1 << 30)
    dev = torch.device("cuda:0")
    wl = args.workload
    res = {"metric": "zero_copy_gather_GBps", "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "data": "synthetic",
           "h2d_peak_GBps": round(h2d_peak, 2), "host": {"cores_visible": ncores, "device": torch.cuda.get_device_name(0)}}

    def pinned(a):
        return torch.from_numpy(a).pin_memory()

    def finish(value, ms_per_step, dtype, config, **more):
        res.update({"value": round(value, 3), "ms_per_step": round(ms_per_step, 4), "dtype": dtype, "config": config,
                    "frac_of_h2d_peak": round(value / h2d_peak, 4)})
        res.update(more)
        print(json.dumps(res))
        return 0

    def spot_check(table, N, D, odtype, ids_np, out, n=2048):
        sample = np.sort(np.random.default_rng(0).choice(ids_np.size, min(n, ids_np.size), replace=False))
        got = out[: ids_np.size * D].view(ids_np.size, D)[torch.from_numpy(sample).to(dev)].cpu().numpy()
        want = np.empty((sample.size, D), dtype=np.uint32)
        oracle.gather_raw(table.host_ptr, N, D, odtype, np.ascontiguousarray(ids_np[sample]), want)
        return bool(np.array_equal(got.view(np.uint32), want))

    if wl == "single":
        N, D, M = 100_000, 128, 16_384
        table = ud.Table(N, D, ud.UD_F32)
        workloads.fill_uniform_f32(table.host_ptr, 0, N * D)
        ids_np = [workloads.indices_uniform(workloads.IDX_STREAM + k, M, N) for k in range(K + W)]
        ids_dev = [torch.from_numpy(a).to(dev) for a in ids_np]
        out = torch.empty(M * D, dtype=torch.float32, device=dev)
        kern = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W)
        ok = spot_check(table, N, D, oracle.F32, ids_np[-1], out)
        wall = _wall_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, [pinned(a) for a in ids_np], out, W)
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
        ok = ok and spot_check(table, N, D, oracle.F32, ids_np[-1], out)
        return finish(nbytes / ks["median_ms"] / 1e6, ks["median_ms"], "f32",
                      {"workload": "single gather: host-pinned fp32 100,000 x 128 (seed 0), 16,384 int64 IDs uniform with replacement"},
                      kernel_only=ks, call_to_sync_incl_id_copy=ws, wall_GBps=round(nbytes / ws["median_ms"] / 1e6, 2),
                      hip_graph_replay_call_to_sync=_stats(gms),
                      same_size_hipMemcpy_GBps=round(same_size, 2),
                      frac_of_same_size_hipMemcpy=round(nbytes / ks["median_ms"] / 1e6 / same_size, 4),
                      rows_per_s=round(M / ks["median_ms"] * 1e3), parity_spot_check=ok)

    if wl == "graphsage":
        p = workloads.PRODUCTS_LIKE
        N, D = p["N"], p["D"]
        table = ud.Table(N, D, ud.UD_F32)
        workloads.fill_uniform_f32(table.host_ptr, 3, N * D)
        offsets, nbr = workloads.zipf_graph_csr(N, p["mean_degree"], p["dmin"], p["alpha"], 3)
        nb = 100
        ids_np = [workloads.sample_csr(offsets, nbr, p["nseeds"], p["fanout"], 33, b) for b in range(nb)]
        del offsets, nbr
        ids_dev = [torch.from_numpy(a).to(dev) for a in ids_np]
        cap = max(a.size for a in ids_np)
        out = torch.empty(cap * D, dtype=torch.float32, device=dev)
        sorted_dev = [torch.from_numpy(np.sort(a)).to(dev) for a in ids_np]      # secondary: the same IDs in ascending order
        kern_sorted = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, sorted_dev[:W] + sorted_dev, out, W)
        del sorted_dev
        kern = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev[:W] + ids_dev, out, W)
        ok = spot_check(table, N, D, oracle.F32, ids_np[-1], out)
        padded = [pinned(a) for a in ids_np]
        wall = _wall_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, padded[:W] + padded, out, W)
        total_bytes = sum(a.size for a in ids_np) * D * 4
        extra = {}
        if not args.no_cpu:
            ctx = ctypes.c_void_p()
            bl.udb_cpu_centric_create(cap * D * 4, ctypes.byref(ctx))
            for name, th, sl in (("plain", threads, 1), ("double_buffered", threads, 4)):
                _cpu_centric(bl, ctx, table.host_ptr, D * 4, ids_np[0], out.data_ptr(), th, sl)
                ms = [_cpu_centric(bl, ctx, table.host_ptr, D * 4, a, out.data_ptr(), th, sl) for a in ids_np[:20]]
                extra[name] = {"GBps": round(sum(a.size for a in ids_np[:20]) * D * 4 / sum(ms) / 1e6, 2), "threads": th}
            bl.udb_cpu_centric_destroy(ctx)
        sizes = [a.size for a in ids_np]
        return finish(total_bytes / sum(kern) / 1e6, sum(kern) / nb, "f32",
                      {"workload": "GraphSAGE-style minibatch gather: 2,400,000 x 100 fp32 host-pinned table, Zipf power-law "
                                   "CSR graph (mean degree 50), 1,024 seeds, fanout [25,10], de-duplicated; 100 batches; one step = one batch",
                       "unique_ids_per_batch": [min(sizes), max(sizes)]},
                      kernel_only=_stats(kern), call_to_sync_incl_id_copy=_stats(wall),
                      sorted_ids_GBps=round(total_bytes / sum(kern_sorted) / 1e6, 2),
                      wall_GBps=round(total_bytes / sum(wall) / 1e6, 2), rows_per_s=round(sum(sizes) / sum(kern) * 1e3),
                      cpu_centric=extra or None, parity_spot_check=ok)

    if wl == "large":
        p = workloads.PAPERS_LIKE
        N, D = 62_500_000, p["D"]       # the largest table the box can pin (111,000,000 rows = 105.9 GiB is refused)
        table = ud.Table(N, D, ud.UD_F32)
        workloads.fill_uniform_f32(table.host_ptr, 4, N * D)
        nb = max(K, 5)
        ids_np = [workloads.sample_procedural(N, p["degree"], p["alpha"], 4, p["nseeds"], p["fanout"], 44, b) for b in range(nb)]
        ids_dev = [torch.from_numpy(a).to(dev) for a in ids_np]
        cap = max(a.size for a in ids_np)
        out = torch.empty(cap * D, dtype=torch.float32, device=dev)
        sorted_dev = [torch.from_numpy(np.sort(a)).to(dev) for a in ids_np]
        kern_sorted = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, sorted_dev[:W] + sorted_dev, out, W)
        del sorted_dev
        kern = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev[:W] + ids_dev, out, W)
        ok = spot_check(table, N, D, oracle.F32, ids_np[-1], out)
        total_bytes = sum(a.size for a in ids_np) * D * 4
        # device-resident variant on a 16,000,000-row slice: IDs folded into the slice, de-duplicated again
        srows = 16_000_000
        devt = table.to_device(0, srows)
        folded = []
        for a in ids_np:
            f = a % srows
            _, first = np.unique(f, return_index=True)
            folded.append(np.ascontiguousarray(f[np.sort(first)]))
        fdev = [torch.from_numpy(a).to(dev) for a in folded]
        kern_h = _kernel_times(ud, torch, devt.device_ptr, srows, D, ud.UD_F32, fdev[:W] + fdev, out, W)
        hbm_bytes = sum(a.size for a in folded) * (2 * D * 4 + 8)
        devt.free()
        sizes = [a.size for a in ids_np]
        return finish(total_bytes / sum(kern) / 1e6, sum(kern) / nb, "f32",
                      {"workload": "large host-resident table: 62,500,000 x 256 fp32 (64 GB pinned; the named 111,000,000 rows "
                                   "exceed what hipHostMalloc grants on this box), procedural Zipf graph, 1,024 seeds, fanout "
                                   "[15,10,5], de-duplicated; one step = one batch", "unique_ids_per_batch": [min(sizes), max(sizes)]},
                      kernel_only=_stats(kern), rows_per_s=round(sum(sizes) / sum(kern) * 1e3),
                      sorted_ids_GBps=round(total_bytes / sum(kern_sorted) / 1e6, 2),
                      device_resident_slice={"rows": srows, "GBps_read_plus_write": round(hbm_bytes / sum(kern_h) / 1e6, 1),
                                             "frac_of_8TBps": round(hbm_bytes / sum(kern_h) / 1e6 / HBM_PEAK_GBPS, 4),
                                             "kernel_only": _stats(kern_h)},
                      parity_spot_check=ok)

    if wl == "hybrid":
        # hot-row cache in HBM on the two graph workloads: the most popular rows are read from HBM,
        # the rest over the host link, in one kernel
        cases = {}
        stream = torch.cuda.current_stream().cuda_stream
        ok = True
        tot_b = tot_ms = 0.0
        for name, p, N, seed, sseed, fracs in (("products_like", workloads.PRODUCTS_LIKE, 2_400_000, 3, 33, (0.01, 0.05, 0.2)),
                                               ("papers_like", workloads.PAPERS_LIKE, 62_500_000, 4, 44, (0.01, 0.05, 0.256))):
            D = p["D"]
            table = ud.Table(N, D, ud.UD_F32)
            workloads.fill_uniform_f32(table.host_ptr, seed, N * D)
            nb = 10
            if "mean_degree" in p:
                offsets, nbr = workloads.zipf_graph_csr(N, p["mean_degree"], p["dmin"], p["alpha"], seed)
                ids_np = [workloads.sample_csr(offsets, nbr, p["nseeds"], p["fanout"], sseed, b) for b in range(nb)]
                del offsets, nbr
            else:
                ids_np = [workloads.sample_procedural(N, p["degree"], p["alpha"], seed, p["nseeds"], p["fanout"], sseed, b)
                          for b in range(nb)]
            ids_dev = [torch.from_numpy(a).to(dev) for a in ids_np]
            out = torch.empty(max(a.size for a in ids_np) * D, dtype=torch.float32, device=dev)
            rows = sum(a.size for a in ids_np)
            useful = rows * D * 4
            plain = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev[:W] + ids_dev, out, W)
            r = {"plain_zero_copy_GBps": round(useful / sum(plain) / 1e6, 2), "caches": {}}
            for frac in fracs:
                n_hot = int(N * frac)
                hot = workloads.hottest_nodes(N, n_hot, seed)
                cache = ud.Cache(table, hot)
                hits = sum(int(np.isin(a, hot[: n_hot]).sum()) if n_hot <= 5_000_000 else -1 for a in ids_np[:1])
                ev = []
                for k, ids in enumerate(ids_dev[:W] + ids_dev):
                    if k >= W:
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                    ud.ud_gather_cached(cache.handle, ud.UD_F32, ids.data_ptr(), ud.UD_I64, ids.numel(), out.data_ptr(), stream)
                    if k >= W:
                        e1.record()
                        ev.append((e0, e1))
                torch.cuda.synchronize()
                ud.ud_gather_status(stream)
                ok = ok and spot_check(table, N, D, oracle.F32, ids_np[-1], out)
                ms = [a.elapsed_time(b) for a, b in ev]
                r["caches"][f"{frac:g}"] = {"rows_cached": n_hot, "hbm_GB": round(n_hot * D * 4 / 1e9 + N * 4 / 1e9, 2),
                                            "effective_GBps": round(useful / sum(ms) / 1e6, 2),
                                            "speedup_vs_plain": round(sum(plain) / sum(ms), 3),
                                            "hit_fraction_batch0": round(hits / ids_np[0].size, 4) if hits >= 0 else None,
                                            "kernel_only": _stats(ms)}
                if frac == fracs[-1]:
                    tot_b += useful
                    tot_ms += sum(ms)
                cache.free()
            cases[name] = r
            table.free()
        return finish(tot_b / tot_ms / 1e6, tot_ms / 20, "f32",
                      {"workload": "hybrid placement: hot-row cache in HBM (most popular rows by rank) over the host-pinned "
                                   "table, on the two GraphSAGE-style workloads; value = useful bytes / time with the "
                                   "largest cache; one step = one batch"},
                      cases=cases, parity_spot_check=ok)

    if wl == "scatter":
        # write direction: rows scattered from HBM into the host-pinned table (distinct IDs)
        best, med = ctypes.c_double(), ctypes.c_double()
        bl.udb_d2h_peak(1 << 30, 10, ctypes.byref(best), ctypes.byref(med))
        d2h_peak = best.value
        N, M = N_ROWS, M_ROWS
        dmax = max(WIDTHS)
        table = ud.Table(N, dmax, ud.UD_F32)
        workloads.fill_uniform_f32(table.host_ptr, 8, N * dmax)
        src = torch.empty(M * dmax, dtype=torch.float32, device=dev).uniform_(-1, 1)
        reps = min(K, 10)
        perms = [np.random.default_rng(k).permutation(N)[:M].astype(np.int64) for k in range(reps + W)]
        ids_dev = [torch.from_numpy(a).to(dev) for a in perms]
        stream = torch.cuda.current_stream().cuda_stream
        devt = table.to_device()
        rows, ok = {}, True
        tot_b = tot_ms = 0.0
        for D in WIDTHS:
            per = {}
            for where, tptr in (("host", table.device_ptr), ("hbm", devt.device_ptr)):
                ev = []
                for k, ids in enumerate(ids_dev):
                    if k >= W:
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                    ud.ud_scatter(tptr, N, D, ud.UD_F32, ids.data_ptr(), ud.UD_I64, M, src.data_ptr(), stream)
                    if k >= W:
                        e1.record()
                        ev.append((e0, e1))
                torch.cuda.synchronize()
                ud.ud_gather_status(stream)
                per[where] = _stats([a.elapsed_time(b) for a, b in ev])
            # spot check on the host table: sampled rows of the last scatter equal their source rows
            samp = np.sort(np.random.default_rng(1).choice(M, 2048, replace=False))
            last = perms[-1]
            want = src[: M * D].view(M, D)[torch.from_numpy(samp).to(dev)].cpu().numpy()
            got = np.empty((samp.size, D), dtype=np.uint32)
            oracle.gather_raw(table.host_ptr, N, D, oracle.F32, np.ascontiguousarray(last[samp]), got)
            ok = ok and bool(np.array_equal(got, want.view(np.uint32)))
            nbytes = M * D * 4
            rows[str(D)] = {"row_bytes": D * 4, "host_ms": per["host"]["median_ms"],
                            "host_GBps": round(nbytes / per["host"]["median_ms"] / 1e6, 2),
                            "frac_of_d2h_peak": round(nbytes / per["host"]["median_ms"] / 1e6 / d2h_peak, 4),
                            "hbm_GBps_read_plus_write": round(2 * nbytes / per["hbm"]["median_ms"] / 1e6, 1)}
            tot_b += nbytes
            tot_ms += per["host"]["median_ms"]
        devt.free()
        res["d2h_peak_GBps"] = round(d2h_peak, 2)
        return finish(tot_b / tot_ms / 1e6, tot_ms, "f32",
                      {"workload": "write direction: 1,000,000 distinct rows scattered from HBM into a host-pinned fp32 table "
                                   "4,000,000 x D, D in {16,64,100,128,256,602}; one step = one scatter per width"},
                      per_width=rows, frac_of_d2h_peak=round(tot_b / tot_ms / 1e6 / d2h_peak, 4), parity_spot_check=ok)

    if wl == "overlap":
        # gather for batch b+1 on a second stream while a stand-in consumer (dense layers on the gathered
        # features) works on batch b: how much of the gather time disappears behind compute
        p = workloads.PAPERS_LIKE
        N, D = 16_000_000, p["D"]
        table = ud.Table(N, D, ud.UD_F32)
        workloads.fill_uniform_f32(table.host_ptr, 4, N * D)
        nb = 12
        ids_np = [workloads.sample_procedural(N, p["degree"], p["alpha"], 4, p["nseeds"], p["fanout"], 44, b) for b in range(nb)]
        M = min(a.size for a in ids_np)
        ids_dev = [torch.from_numpy(np.ascontiguousarray(a[:M])).to(dev) for a in ids_np]
        bufs = [torch.empty((M, D), dtype=torch.float32, device=dev) for _ in range(2)]
        hidden = 1024
        w1 = torch.randn(D, hidden, device=dev) * 0.05
        w2 = torch.randn(hidden, hidden, device=dev) * 0.05
        layers = 1

        consumer = {"kind": "gemm"}
        scratch = torch.empty((M, D), dtype=torch.float32, device=dev)

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
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3

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

        variants = {}
        for name, tun in (("auto_512wg", None), ("256wg", ud.ud_tuning(0, 0, 0, 256, 0)),
                          ("128wg", ud.ud_tuning(0, 0, 0, 128, 0)), ("64wg", ud.ud_tuning(0, 0, 0, 64, 0)),
                          ("64wg_4rows_in_flight", ud.ud_tuning(0, 1, 4, 64, 0)),
                          ("32wg_4rows_in_flight", ud.ud_tuning(0, 1, 4, 32, 0)),
                          ("share_gpu_flag", ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_SHARE_GPU)),
                          ("32wg_of_1024", ud.ud_tuning(0, 0, 0, 32, ud.UD_TUNE_BIG_BLOCKS)),
                          ("16wg_of_1024", ud.ud_tuning(0, 0, 0, 16, ud.UD_TUNE_BIG_BLOCKS)),
                          ("16wg_of_1024_2rows", ud.ud_tuning(0, 1, 2, 16, ud.UD_TUNE_BIG_BLOCKS)),
                          ("8wg_of_1024_2rows", ud.ud_tuning(0, 1, 2, 8, ud.UD_TUNE_BIG_BLOCKS)),
                          ("8wg_of_1024_4rows", ud.ud_tuning(0, 1, 4, 8, ud.UD_TUNE_BIG_BLOCKS))):
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
        for name, tun in (("auto_512wg", None), ("128wg", ud.ud_tuning(0, 0, 0, 128, 0)), ("64wg", ud.ud_tuning(0, 0, 0, 64, 0)),
                          ("share_gpu_flag", ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_SHARE_GPU))):
            tg = timed(only_gather(tun)) / nb
            to = timed(overlapped(tun)) / nb
            elementwise[name] = {"gather_only_ms": round(tg, 3), "overlapped_ms": round(to, 3),
                                 "gather_ms_while_overlapped": round(spans["gather"], 3),
                                 "compute_ms_while_overlapped": round(spans["compute"], 3),
                                 "hidden_fraction_of_gather": round(1.0 - max(to - t_e, 0.0) / tg, 3)}
        consumer["kind"] = "gemm"
        ud.ud_gather_status(sg.cuda_stream)
        ok = spot_check(table, N, D, oracle.F32, np.ascontiguousarray(ids_np[nb - 1][:M]), bufs[(nb - 1) & 1].view(-1))
        best = min(variants.values(), key=lambda v: v["overlapped_ms"])
        return finish(M * D * 4 / best["overlapped_ms"] / 1e6, best["overlapped_ms"], "f32",
                      {"workload": f"overlap: zero-copy gather of batch b+1 ({M} rows x 1024 B from a 16,000,000-row host table) "
                                   f"on one stream while {layers + 1} dense fp32 layers (hidden {hidden}) consume batch b on another; "
                                   "value = gathered bytes / per-batch time of the overlapped pipeline"},
                      compute_only_ms=round(t_c, 3), variants=variants, elementwise_consumer=elementwise,
                      parity_spot_check=ok)

    if wl == "padded":
        # the same gathers from tables whose row pitch is rounded up to 128 bytes (UD_TABLE_PAD_ROWS):
        # no row shares a memory line with its neighbours, so nothing but the row's own lines is fetched
        N, M = N_ROWS, M_ROWS
        stream = torch.cuda.current_stream().cuda_stream
        reps = min(K, 10)
        cases, ok = {}, True
        tot_b = tot_ms = 0.0
        for name, elem, dtype, odtype, D in (("f32_D100", ud.UD_F32, ud.UD_F32, oracle.F32, 100),
                                             ("f32_D602", ud.UD_F32, ud.UD_F32, oracle.F32, 602),
                                             ("f16_to_f32_D602", ud.UD_F16, ud.UD_F16_TO_F32, oracle.F16_TO_F32, 602)):
            esz = 4 if elem == ud.UD_F32 else 2
            ids_np = [workloads.indices_uniform(workloads.IDX_STREAM + k, M, N) for k in range(reps + W)]
            ids_dev = [torch.from_numpy(a).to(dev) for a in ids_np]
            out = torch.empty(M * D, dtype=torch.float32, device=dev)
            r = {}
            for kind, flags in (("dense", 0), ("padded", ud.UD_TABLE_PAD_ROWS)):
                t = ud.Table(N, D, elem, flags)
                if elem == ud.UD_F32:
                    workloads.fill_uniform_f32(t.host_ptr, 9, N * t.pitch)
                else:
                    workloads.fill_normal_f16(t.host_ptr, 9, N * t.pitch)
                ev = []
                for k, ids in enumerate(ids_dev):
                    if k >= W:
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                    ud.ud_gather_pitched(t.device_ptr, N, D, t.pitch, dtype, ids.data_ptr(), ud.UD_I64, M, out.data_ptr(), stream)
                    if k >= W:
                        e1.record()
                        ev.append((e0, e1))
                torch.cuda.synchronize()
                ud.ud_gather_status(stream)
                st = _stats([a.elapsed_time(b) for a, b in ev])
                samp = np.sort(np.random.default_rng(0).choice(M, 2048, replace=False))
                got = out.view(M, D)[torch.from_numpy(samp).to(dev)].cpu().numpy()
                want = np.empty((samp.size, D), dtype=np.uint32)
                oracle.gather_raw(t.host_ptr, N, D, odtype, np.ascontiguousarray(ids_np[-1][samp]), want, pitch=t.pitch)
                ok = ok and bool(np.array_equal(got.view(np.uint32), want))
                useful = M * D * esz
                r[kind] = {"pitch_bytes": t.pitch * esz, "ms": st["median_ms"], "GBps": round(useful / st["median_ms"] / 1e6, 2),
                           "frac_of_h2d_peak": round(useful / st["median_ms"] / 1e6 / h2d_peak, 4),
                           "table_GB": round(t.nbytes / 1e9, 2)}
                if kind == "padded":
                    tot_b += useful
                    tot_ms += st["median_ms"]
                t.free()
            r["speedup"] = round(r["dense"]["ms"] / r["padded"]["ms"], 3)
            cases[name] = r
        return finish(tot_b / tot_ms / 1e6, tot_ms, "f32",
                      {"workload": "padded rows: 1,000,000 int64 IDs from 4,000,000-row host-pinned tables with the row pitch "
                                   "rounded up to 128 bytes, against the dense layout; value = useful bytes / time, padded tables"},
                      cases=cases, parity_spot_check=ok)

    if wl == "fp16":
        N, D, M = 10_000_000, 602, 2_000_000
        table = ud.Table(N, D, ud.UD_F16)
        workloads.fill_normal_f16(table.host_ptr, 5, N * D)
        ids_np = [workloads.indices_uniform(workloads.IDX_STREAM + k, M, N, np.int32) for k in range(min(K, 10) + W)]
        ids_dev = [torch.from_numpy(a).to(dev) for a in ids_np]
        out = torch.empty(M * D, dtype=torch.float32, device=dev)
        kern = _kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F16_TO_F32, ids_dev, out, W)
        ok = spot_check(table, N, D, oracle.F16_TO_F32, ids_np[-1], out)
        ks = _stats(kern)
        link_bytes = M * D * 2
        return finish(link_bytes / ks["median_ms"] / 1e6, ks["median_ms"], "f16->f32",
                      {"workload": "half-precision odd-width table: host-pinned fp16 10,000,000 x 602 (N(0,1) rounded to fp16), "
                                   "2,000,000 int32 IDs uniform, fused upcast to fp32 in HBM"},
                      kernel_only=ks, hbm_write_GBps=round(2 * link_bytes / ks["median_ms"] / 1e6, 2),
                      rows_per_s=round(M / ks["median_ms"] * 1e3), parity_spot_check=ok)

    if wl == "align":
        # Section 5.3 / Figure 7 of the paper: row sizes 2048..2076 bytes in 4-byte steps
        N, M = 4_000_000, 262_144
        widths = list(range(512, 520))
        dmax = widths[-1]
        table = ud.Table(N, dmax, ud.UD_F32)
        workloads.fill_uniform_f32(table.host_ptr, 7, N * dmax)
        reps = max(K, 5)
        ids_np = [workloads.indices_uniform(workloads.IDX_STREAM + k, M, N) for k in range(reps + W)]
        ids_dev = [torch.from_numpy(a).to(dev) for a in ids_np]
        out = torch.empty(M * dmax, dtype=torch.float32, device=dev)
        ctx = ctypes.c_void_p()
        bl.udb_cpu_centric_create(M * dmax * 4, ctypes.byref(ctx))
        naive = ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_ELEMENTWISE)
        shifted = ud.ud_tuning(0, 0, 0, 0, ud.UD_TUNE_ELEMENTWISE | ud.UD_TUNE_CIRCULAR_SHIFT)
        rows, ok = {}, True
        for D in widths:
            nbytes = M * D * 4
            opt = _stats(_kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W))
            ok = ok and spot_check(table, N, D, oracle.F32, ids_np[-1], out)
            nv = _stats(_kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W, naive))
            sh = _stats(_kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W, shifted))
            _cpu_centric(bl, ctx, table.host_ptr, D * 4, ids_np[0], out.data_ptr(), threads)
            py = sorted(_cpu_centric(bl, ctx, table.host_ptr, D * 4, a, out.data_ptr(), threads) for a in ids_np[1:6])[2]
            rows[str(D * 4)] = {"zero_copy_ms": opt["median_ms"], "zero_copy_GBps": round(nbytes / opt["median_ms"] / 1e6, 2),
                                "one_lane_per_element_ms": nv["median_ms"],
                                "one_lane_per_element_GBps": round(nbytes / nv["median_ms"] / 1e6, 2),
                                "circular_shift_ms": sh["median_ms"],
                                "circular_shift_GBps": round(nbytes / sh["median_ms"] / 1e6, 2),
                                "cpu_centric_ms": round(py, 4), "ideal_ms": round(nbytes / h2d_peak / 1e6, 4),
                                "speedup_vs_cpu_centric": round(py / opt["median_ms"], 3),
                                "one_lane_per_element_speedup_vs_cpu_centric": round(py / nv["median_ms"], 3)}
        bl.udb_cpu_centric_destroy(ctx)
        tot_b = sum(M * D * 4 for D in widths)
        tot_ms = sum(r["zero_copy_ms"] for r in rows.values())
        return finish(tot_b / tot_ms / 1e6, tot_ms, "f32",
                      {"workload": "alignment sweep: host-pinned fp32 table 4,000,000 rows, row bytes 2048..2076 step 4, "
                                   "262,144 int64 IDs uniform; one step = one gather per row size", "cpu_centric_threads": threads},
                      per_row_bytes=rows, parity_spot_check=ok)

    if wl == "grid":
        # Section 5.2 / Figure 6 of the paper: (rows copied, row bytes) from (8K, 256B) to (256K, 16KB)
        region = 16 << 30
        table = ud.Table(region // 16384, 4096, ud.UD_F32)      # 16 GiB, viewed with each row size
        workloads.fill_uniform_f32(table.host_ptr, 6, region // 4)
        reps = max(K, 5)
        ctx = ctypes.c_void_p()
        bl.udb_cpu_centric_create(262_144 * 16384, ctypes.byref(ctx))
        out = torch.empty(262_144 * 4096, dtype=torch.float32, device=dev)
        cells, ok = {}, True
        tot_b = tot_ms = 0.0
        for rb in (256, 1024, 4096, 16384):
            D, N = rb // 4, region // rb
            for M in (8_192, 32_768, 131_072, 262_144):
                ids_np = [workloads.indices_uniform(workloads.IDX_STREAM + k, M, N) for k in range(reps + W)]
                ids_dev = [torch.from_numpy(a).to(dev) for a in ids_np]
                nbytes = M * rb
                kern = _stats(_kernel_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, ids_dev, out, W))
                ok = ok and spot_check(table, N, D, oracle.F32, ids_np[-1], out, 512)
                wall = _stats(_wall_times(ud, torch, table.device_ptr, N, D, ud.UD_F32, [pinned(a) for a in ids_np], out, W))
                _cpu_centric(bl, ctx, table.host_ptr, rb, ids_np[0], out.data_ptr(), threads)
                py = sorted(_cpu_centric(bl, ctx, table.host_ptr, rb, a, out.data_ptr(), threads) for a in ids_np[1:6])[2]
                ideal = nbytes / h2d_peak / 1e6
                cells[f"({M // 1024}K, {rb}B)"] = {
                    "MB": round(nbytes / 1e6, 2), "kernel_ms": kern["median_ms"], "call_to_sync_ms": wall["median_ms"],
                    "cpu_centric_ms": round(py, 4), "ideal_ms": round(ideal, 4),
                    "slowdown_vs_ideal": round(wall["median_ms"] / ideal, 3),
                    "cpu_centric_slowdown_vs_ideal": round(py / ideal, 3),
                    "speedup_vs_cpu_centric": round(py / wall["median_ms"], 3)}
                tot_b += nbytes
                tot_ms += kern["median_ms"]
        bl.udb_cpu_centric_destroy(ctx)
        return finish(tot_b / tot_ms / 1e6, tot_ms, "f32",
                      {"workload": "size grid: 16 GiB host-pinned fp32 region viewed as rows of 256 B..16 KB, "
                                   "8K..256K int64 IDs uniform; call-to-sync times include the ID list's H2D copy; "
                                   "one step = one gather per cell", "cpu_centric_threads": threads},
                      cells=cells, parity_spot_check=ok)
    raise ValueError(wl)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--threads", type=int, default=0, help="host threads of the CPU-centric baseline (0 = all)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the host baselines (for profiling runs)")
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
    if args.workload != "sweep":
        return run_other(args, ud, bl, workloads, torch, np, threads, ncores)

    # ---- host-link peak: best of 10 pinned hipMemcpy H2D of 1 GiB, same process ----
    best, med = ctypes.c_double(), ctypes.c_double()
    if bl.udb_h2d_peak(1 << 30, 10, ctypes.byref(best), ctypes.byref(med)) != 0:
        raise RuntimeError("host-link peak measurement failed")
    h2d_peak = best.value
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
    traffic = _read_traffic_note()
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
                     "frac": round(dom_achieved / h2d_peak, 4), "traffic": traffic,
                     "traffic_unit": "bytes per launch (L2<->fabric reads + writes, rocprofv3 FETCH_SIZE/WRITE_SIZE)",
                     "algorithmic_bytes_per_launch": M_ROWS * (2 * 602 * 4 + 8),
                     "link_bytes_per_launch": M_ROWS * 602 * 4,
                     # a dense table of 2408-byte rows makes a row overlap 19.75 128-byte lines on average (the
                     # hardware fetches whole lines): the most a gather of this layout can show is 2408 / 2528 of the peak
                     "line_floor_bytes_per_launch": int(M_ROWS * 19.75 * 128),
                     "frac_incl_line_padding": round(M_ROWS * 19.75 * 128 / dom_ms / 1e6 / h2d_peak, 4),
                     "peak_source": "best of 10 pinned hipMemcpy H2D of 1 GiB in this run",
                     "ms_per_launch": round(dom_ms, 4)},
        "roofline_hbm": {"bound": "hbm", "kernel": "gather_chunked<f32> D=602, table in HBM",
                         "achieved": round(hbm_achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": round(hbm_achieved / HBM_PEAK_GBPS, 4),
                         "traffic": _read_traffic_note("hbm_variant_traffic_bytes_per_launch"),
                         "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE)",
                         "algorithmic_bytes_per_launch": hbm_bytes_602,
                         "per_width_GBps_read_plus_write": {str(D): round(M_ROWS * (2 * D * 4 + 8) / per_ms_hbm[D] / 1e6, 1)
                                                            for D in WIDTHS},
                         "ms_per_launch": round(per_ms_hbm[602], 4),
                         "sweep_GBps_read_plus_write": round(K * 2 * bytes_per_step / elapsed_hbm / 1e9, 1),
                         "d2d_memcpy_traffic_GBps": round(2 * d2d_copy, 1)},
        "cpu_baseline": cpu_baseline,
        "cpu_centric": cpu_centric,
        "host": {"cores_visible": ncores, "device": torch.cuda.get_device_name(0), **_host_topology()},
    }
    table.free()
    print(json.dumps(line))
    return 0 if parity_ok else 1


if __name__ == "__main__":
    sys.exit(main())
