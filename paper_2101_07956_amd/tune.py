"""Tuning loop for the row gather: sweeps the launch parameters of ``ud_gather_tuned`` on the GPU
that is present, for a host-pinned table and for its HBM-resident copy, and reports each shape's
rate against the roofline that bounds it -- the pinned ``hipMemcpy`` peak measured in the same
run for the host link, the chip's published HBM peak for the device-resident variant.

    python -m paper_2101_07956_amd.tune --widths 16,64,100,128,256,602 --rows 1000000 --table-rows 4000000

prints, per width and residence, the best shapes, the shape ``ud_gather`` picks by itself, and how
far apart they are; ``--json FILE`` also writes every measurement.

    python -m paper_2101_07956_amd.tune --amplification prof_fetch/fetch_counter_collection.csv \
        --rows 1000000 --scale 2.0

turns a ``rocprofv3 --pmc FETCH_SIZE`` (or ``WRITE_SIZE``) counter file of a ``bench.py`` run into bytes
moved per launch of every gather kernel; ``--scale`` is the factor that makes the counter read the
known size of the plain 1 GiB copy kernel the benchmark runs first (the tool prints that reading).

The automatic plan in ``csrc/ud_boundary.hip`` was set from this loop's output on MI355X.
"""
from __future__ import annotations

import argparse
import csv
import ctypes
import json
import os
import sys

HBM_PEAK_GBPS = 8000.0


def _amplification(path: str, scale: float) -> int:
    per = {}
    copy = None
    for r in csv.DictReader(open(path)):
        name, val = r["Kernel_Name"], float(r["Counter_Value"])
        if "plain_copy_kernel" in name:
            copy = val
        if "gather_chunked" in name or "gather_elementwise" in name or "scatter_chunked" in name:
            short = name.replace("void ud::", "").replace("(ud::GatherArgs, int)", "").replace("(ud::GatherArgs)", "")
            per.setdefault((short, r["Grid_Size"], r["Counter_Name"]), []).append(val)
    if copy is not None:
        print(f"plain 1 GiB copy kernel reads {copy:.0f} KiB on this counter -> scale {1048576.0 / copy:.4f}")
    print(f"{'kernel':44s} {'grid':>10s} {'counter':>11s} {'launches':>8s} {'MB per launch':>14s}")
    for (k, g, c), v in per.items():
        print(f"{k:44s} {g:>10s} {c:>11s} {len(v):8d} {sum(v) / len(v) * scale * 1024 / 1e6:14.1f}")
    return 0


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--widths", default="16,64,100,128,256,602", help="row widths in fp32 elements")
    ap.add_argument("--rows", type=int, default=1_000_000, help="rows gathered per launch")
    ap.add_argument("--table-rows", type=int, default=4_000_000)
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--top", type=int, default=5)
    ap.add_argument("--json", default=None)
    ap.add_argument("--amplification", default=None, help="rocprofv3 counter_collection.csv to summarise instead of sweeping")
    ap.add_argument("--scale", type=float, default=1.0)
    args = ap.parse_args()
    if args.amplification:
        return _amplification(args.amplification, args.scale)

    import numpy as np
    import torch

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    if root not in sys.path:
        sys.path.insert(0, root)
    import paper_2101_07956_amd as ud
    import workloads

    widths = [int(x) for x in args.widths.split(",")]
    N, M, dmax = args.table_rows, args.rows, max(widths)
    bl = ctypes.CDLL(os.path.join(os.path.dirname(ud.LIB_PATH), "libud_baseline.so"))
    dp = ctypes.POINTER(ctypes.c_double)
    bl.udb_h2d_peak.argtypes = [ctypes.c_size_t, ctypes.c_int, dp, dp]
    best, med = ctypes.c_double(), ctypes.c_double()
    bl.udb_h2d_peak(1 << 30, 10, ctypes.byref(best), ctypes.byref(med))
    h2d = best.value
    print(f"{torch.cuda.get_device_name(0)}: pinned hipMemcpy H2D peak {h2d:.2f} GB/s; HBM peak taken as {HBM_PEAK_GBPS:.0f} GB/s")

    table = ud.Table(N, dmax, ud.UD_F32)
    workloads.fill_uniform_f32(table.host_ptr, 1, N * dmax)
    dev_table = table.to_device()
    idx = torch.from_numpy(workloads.indices_uniform(workloads.IDX_STREAM, M, N)).cuda()
    out = torch.empty(M * dmax, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def rate(tptr, D, tun, useful):
        ud.ud_gather_tuned(tptr, N, D, ud.UD_F32, idx.data_ptr(), ud.UD_I64, M, out.data_ptr(), stream, tun)
        ts = []
        for _ in range(args.reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ud.ud_gather_tuned(tptr, N, D, ud.UD_F32, idx.data_ptr(), ud.UD_I64, M, out.data_ptr(), stream, tun)
            e1.record()
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return useful / sorted(ts)[len(ts) // 2] / 1e6

    shapes = [(u, p) for u in (1, 2, 4) for p in (1, 2, 3, 4) if u * p <= 8 and (u, p) != (4, 2)]
    everything = []
    for where, tptr, peak in (("host", table.device_ptr, h2d), ("hbm", dev_table.device_ptr, HBM_PEAK_GBPS)):
        for D in widths:
            useful = M * D * 4 * (1 if where == "host" else 2)      # link bytes, or HBM read + write
            chunks = (D * 4 + 15) // 16
            natural = 1
            while natural < chunks and natural < 64:
                natural *= 2
            res = []
            for lanes in sorted({natural, min(64, natural * 2), 64}):
                for u, p in shapes:
                    for blocks in (128, 512, 2048, 0):
                        for flags in ((0, ud.UD_TUNE_NT_STORE) if where == "hbm" else (0,)):
                            g = rate(tptr, D, ud.ud_tuning(lanes, p, u, blocks, flags), useful)
                            res.append({"GBps": round(g, 2), "lanes": lanes, "rows_in_flight": u, "chunks_per_lane": p,
                                        "max_blocks": blocks, "flags": flags})
            res.sort(key=lambda r: -r["GBps"])
            auto_plan = ud.ud_gather_plan(tptr, D, ud.UD_F32)
            auto = rate(tptr, D, None, useful)
            print(f"[{where}] D={D} ({D * 4} B rows): automatic plan lanes={auto_plan.lanes_per_row} "
                  f"rows_in_flight={auto_plan.rows_in_flight} chunks_per_lane={auto_plan.chunks_per_lane} "
                  f"max_blocks={auto_plan.max_blocks} flags={auto_plan.flags}: {auto:.2f} GB/s = {100 * auto / peak:.1f}% of peak; "
                  f"best swept {res[0]['GBps']:.2f} ({100 * res[0]['GBps'] / peak:.1f}%)")
            for r in res[: args.top]:
                print(f"      {r['GBps']:9.2f} GB/s  lanes={r['lanes']:2d} rows_in_flight={r['rows_in_flight']} "
                      f"chunks_per_lane={r['chunks_per_lane']} max_blocks={r['max_blocks']} flags={r['flags']}")
            everything.append({"table": where, "D": D, "automatic_GBps": round(auto, 2), "peak_GBps": round(peak, 2), "sweep": res})
    ud.ud_gather_status(stream)
    if args.json:
        with open(args.json, "w") as f:
            json.dump(everything, f)
    dev_table.free()
    table.free()
    return 0


if __name__ == "__main__":
    sys.exit(main())
