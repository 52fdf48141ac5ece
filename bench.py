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
    bl.udb_plain_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    bl.udb_cpu_centric_create.argtypes = [ctypes.c_size_t, ctypes.POINTER(ctypes.c_void_p)]
    bl.udb_cpu_centric_destroy.argtypes = [ctypes.c_void_p]
    bl.udb_cpu_centric_gather.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                          ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, dp, dp, dp]
    return bl


def _read_traffic_note():
    """Fabric traffic (bytes per launch) of the dominant kernel, measured offline with rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE and kept in the committed counter summary; None if that file is absent."""
    path = os.path.join(ROOT, "profiles", "gather_f32_D602_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch="):
            return float(line.split("=", 1)[1])
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--threads", type=int, default=0, help="host threads of the CPU-centric baseline (0 = all)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the host baselines (for profiling runs)")
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
    import paper_2101_07956_amd as ud
    import workloads

    bl = _load_baseline_lib(ud)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    K, W = args.steps, args.warmup
    ncores = len(os.sched_getaffinity(0))
    threads = args.threads or min(ncores, 16)

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
        per = {D: sum(a.elapsed_time(b) for a, b in ev) / len(ev) for D, ev in events.items()}   # ms per launch
        return elapsed, per

    elapsed, per_ms = timed(table.device_ptr)
    bytes_per_step = sum(M_ROWS * D * 4 for D in WIDTHS)
    value = K * bytes_per_step / elapsed / 1e9
    rows_per_s = K * M_ROWS * len(WIDTHS) / elapsed
    per_width = {
        str(D): {"row_bytes": D * 4, "ms": round(per_ms[D], 4), "GBps": round(M_ROWS * D * 4 / per_ms[D] / 1e6, 2),
                 "frac_of_h2d_peak": round(M_ROWS * D * 4 / per_ms[D] / 1e6 / h2d_peak, 4),
                 "rows_per_s": round(M_ROWS / per_ms[D] * 1e3)}
        for D in WIDTHS
    }

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
        # oracle: one full step (six widths x 1,000,000 rows), single thread
        obuf = np.empty(M_ROWS * dmax, dtype=np.uint32)
        t0 = time.perf_counter()
        for D in WIDTHS:
            oracle.gather_raw(table.host_ptr, N_ROWS, D, oracle.F32, ids_host[0], obuf[: M_ROWS * D].reshape(M_ROWS, D))
        t_oracle = time.perf_counter() - t0
        cpu_baseline = {"value": round(bytes_per_step / t_oracle / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
                        "sample": "1 step = 6 widths x 1,000,000 rows (4.664 GB gathered)",
                        "seconds": round(t_oracle, 2), "rows_per_s": round(M_ROWS * len(WIDTHS) / t_oracle)}
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
        "rows_per_s": round(rows_per_s),
        "h2d_peak_GBps": round(h2d_peak, 2),
        "per_width": per_width,
        "parity_spot_check": parity_ok,
        "roofline": {"bound": "host_link", "kernel": "gather_chunked<f32> D=602 (2408-byte rows)",
                     "achieved": round(dom_achieved, 2), "peak": round(h2d_peak, 2), "unit": "GB/s",
                     "frac": round(dom_achieved / h2d_peak, 4), "traffic": traffic,
                     "traffic_unit": "bytes per launch (L2<->fabric reads + writes, rocprofv3 FETCH_SIZE/WRITE_SIZE)",
                     "algorithmic_bytes_per_launch": M_ROWS * (2 * 602 * 4 + 8),
                     "link_bytes_per_launch": M_ROWS * 602 * 4,
                     "peak_source": "best of 10 pinned hipMemcpy H2D of 1 GiB in this run",
                     "ms_per_launch": round(dom_ms, 4)},
        "roofline_hbm": {"bound": "hbm", "kernel": "gather_chunked<f32> D=602, table in HBM",
                         "achieved": round(hbm_achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": round(hbm_achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                         "ms_per_launch": round(per_ms_hbm[602], 4),
                         "sweep_GBps_read_plus_write": round(K * 2 * bytes_per_step / elapsed_hbm / 1e9, 1),
                         "d2d_memcpy_traffic_GBps": round(2 * d2d_copy, 1)},
        "cpu_baseline": cpu_baseline,
        "cpu_centric": cpu_centric,
        "host": {"cores_visible": ncores, "device": torch.cuda.get_device_name(0)},
    }
    table.free()
    print(json.dumps(line))
    return 0 if parity_ok else 1


if __name__ == "__main__":
    sys.exit(main())
