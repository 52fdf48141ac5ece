"""Tuning loop for the row gather.

Sweep: the launch parameters of ``ud_gather_tuned`` on the GPU that is present, for a host-pinned table and
for its HBM-resident copy, each shape's rate against the roofline that bounds it -- the pinned
``hipMemcpy`` peak measured in the same run for the host link, the chip's published HBM peak for the
device-resident variant.

    python3 -m paper_2101_07956_amd.tune --widths 16,64,100,128,256,602 --rows 1000000 --table-rows 4000000

prints, per width and residence, the best shapes, the shape ``ud_gather`` picks by itself, and how far apart
they are; ``--json FILE`` also writes every measurement.

Replay: a fixed list of launch shapes -- every kernel the library ships, at the launch shape the library
picks (or a named alternative) -- each launched the same few times, so that hardware counters collected
by a profiler can be attributed to shapes by dispatch order:

    python3 -m paper_2101_07956_amd.tune --replay --json gpurun_out/replay_timing.json          # HIP-event times
    rocprofv3 --pmc FETCH_SIZE -f csv -d gpurun_out/replay_fetch -o fetch -- python3 -m paper_2101_07956_amd.tune --replay
    rocprofv3 --pmc WRITE_SIZE -f csv -d gpurun_out/replay_write -o write -- python3 -m paper_2101_07956_amd.tune --replay
    rocprofv3 --pmc TCC_EA0_RDREQ_sum TCC_EA0_RDREQ_128B_sum TCC_EA0_RDREQ_IO_CREDIT_STALL_sum TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum \
        -f csv -d gpurun_out/replay_req -o req -- python3 -m paper_2101_07956_amd.tune --replay

(one counter set per run; ``python3`` directly after ``--``).  The replay starts with a plain 1 GiB copy
kernel of known size, which is what the byte counters are scaled by.

Summarise: merge the timing file and any number of such counter files into one table, one row per shape:
rate, fraction of the peak that bounds it, bytes fetched and written per launch against the algorithmic
bytes and against the 128-byte-line floor of the layout, read requests per row, credit stalls:

    python3 -m paper_2101_07956_amd.tune --summarise gpurun_out/replay_timing.json gpurun_out/replay_*/*/*counter_collection.csv

Kernel statistics: condense what ``rocprofv3 --kernel-trace --stats`` wrote for a benchmark run (per kernel,
and per kernel and grid size, since several widths share one kernel):

    rocprofv3 --kernel-trace --stats -f csv -d gpurun_out/prof_stats -o stats -- python3 bench.py --headline-only --no-cpu
    python3 -m paper_2101_07956_amd.tune --kernel-stats gpurun_out/prof_stats/stats_kernel_stats.csv gpurun_out/prof_stats/stats_kernel_trace.csv

``--amplification FILE`` is the older single-counter summary of a ``bench.py`` run.

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


KERNEL_MARKS = ("gather_chunked", "gather_flat", "gather_elementwise", "scatter_chunked", "scatter_flat")
REPLAY_LAUNCHES = 3          # per shape: the first is a warm-up, counters are read from the last


def _mean_lines_per_row(row_bytes: int, line: int = 128) -> float:
    """Mean number of `line`-byte lines a row of a dense table (16-byte aligned base) overlaps."""
    import math
    period = line // math.gcd(row_bytes, line)
    return sum(((r * row_bytes) % line + row_bytes + line - 1) // line for r in range(period)) / period


def replay_shapes(ud):
    """(name, kind, dtype, D, residence, ids, tuning) for every shipped kernel at the shape the library picks,
    plus the alternatives worth a row of the table."""
    T = ud.ud_tuning
    NT, DA, EL, CS = ud.UD_TUNE_NT_STORE, ud.UD_TUNE_DEST_ALIGNED, ud.UD_TUNE_ELEMENTWISE, ud.UD_TUNE_CIRCULAR_SHIFT
    shapes = []
    for D in (16, 32, 64, 100, 128, 256, 602):
        shapes.append((f"gather host f32 D={D} auto", "gather", ud.UD_F32, D, "host", "uniform", None))
    for D in (16, 32):
        # same rows-per-second question, asked with page-local IDs: every 4th row in ascending order (no two
        # rows share a 128-byte line or are adjacent lines, consecutive rows share 4 KiB pages)
        shapes.append((f"gather host f32 D={D} auto, IDs 0,4,8,...", "gather", ud.UD_F32, D, "host", "stride4", None))
        shapes.append((f"gather host f32 D={D} auto, IDs sorted", "gather", ud.UD_F32, D, "host", "sorted", None))
    shapes.append(("gather host f32 D=16 lanes=4 rows_in_flight=4", "gather", ud.UD_F32, 16, "host", "uniform", T(4, 1, 4, 0, 0)))
    shapes.append(("gather host f32 D=16 lanes=64 (one row per instruction)", "gather", ud.UD_F32, 16, "host", "uniform", T(64, 1, 1, 0, 0)))
    for D in (16, 64, 100, 128, 256, 602):
        shapes.append((f"gather hbm f32 D={D} auto", "gather", ud.UD_F32, D, "hbm", "uniform", None))
    for D in (100, 256, 602):
        shapes.append((f"gather hbm f32 D={D} source-aligned kernel", "gather", ud.UD_F32, D, "hbm", "uniform", T(0, 0, 0, 0, NT)))
    shapes.append(("gather host f16->f32 D=602 auto", "gather", ud.UD_F16_TO_F32, 602, "host", "uniform", None))
    shapes.append(("gather hbm f16->f32 D=602 auto", "gather", ud.UD_F16_TO_F32, 602, "hbm", "uniform", None))
    shapes.append(("gather host f16 D=602 auto", "gather", ud.UD_F16, 602, "host", "uniform", None))
    shapes.append(("gather host f32 D=513 one lane per element", "gather", ud.UD_F32, 513, "host", "uniform", T(0, 0, 0, 0, EL)))
    shapes.append(("gather host f32 D=513 one lane per element + circular shift", "gather", ud.UD_F32, 513, "host", "uniform", T(0, 0, 0, 0, EL | CS)))
    shapes.append(("gather host f32 D=513 auto", "gather", ud.UD_F32, 513, "host", "uniform", None))
    shapes.append(("cached gather host f32 D=602, 25% of rows in HBM", "cached", ud.UD_F32, 602, "host", "uniform", None))
    for where in ("host", "hbm"):
        for D in (16, 100, 128, 602):
            shapes.append((f"scatter {where} f32 D={D} auto", "scatter", ud.UD_F32, D, where, "perm", None))
    for D in (100, 602):
        shapes.append((f"scatter hbm f32 D={D} row-per-lane-group kernel", "scatter", ud.UD_F32, D, "hbm", "perm", T(0, 0, 0, 0, 0)))
    shapes.append(("scatter hbm f32 D=96 auto (384-byte rows: whole lines)", "scatter", ud.UD_F32, 96, "hbm", "perm", None))
    # row ends on 32-byte and on 64-byte boundaries, with and without streaming stores
    FS = ud.UD_TUNE_FLAT_SOURCE
    shapes.append(("scatter hbm f32 D=104 auto (416-byte rows)", "scatter", ud.UD_F32, 104, "hbm", "perm", None))
    shapes.append(("scatter hbm f32 D=112 auto (448-byte rows)", "scatter", ud.UD_F32, 112, "hbm", "perm", None))
    shapes.append(("scatter hbm f32 D=112 same kernel, ordinary stores", "scatter", ud.UD_F32, 112, "hbm", "perm", T(0, 1, 0, 0, FS)))
    shapes.append(("scatter hbm f32 D=100 same kernel, ordinary stores", "scatter", ud.UD_F32, 100, "hbm", "perm", T(0, 1, 0, 0, FS)))
    return shapes


def _replay(args) -> int:
    import numpy as np
    import torch

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    if root not in sys.path:
        sys.path.insert(0, root)
    import paper_2101_07956_amd as ud
    import workloads

    N, M, dmax = args.table_rows, args.rows, 602
    bl = ctypes.CDLL(os.path.join(os.path.dirname(ud.LIB_PATH), "libud_baseline.so"))
    dp = ctypes.POINTER(ctypes.c_double)
    bl.udb_h2d_peak.argtypes = [ctypes.c_size_t, ctypes.c_int, dp, dp]
    bl.udb_d2h_peak.argtypes = [ctypes.c_size_t, ctypes.c_int, dp, dp]
    bl.udb_plain_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    best, med = ctypes.c_double(), ctypes.c_double()
    bl.udb_h2d_peak(1 << 30, 5, ctypes.byref(best), ctypes.byref(med))
    h2d = best.value
    bl.udb_d2h_peak(1 << 30, 5, ctypes.byref(best), ctypes.byref(med))
    d2h = best.value

    tables = {}
    f32 = ud.Table(N, dmax, ud.UD_F32)
    workloads.fill_uniform_f32(f32.host_ptr, 1, N * dmax)
    f16 = ud.Table(N, dmax, ud.UD_F16)
    workloads.fill_normal_f16(f16.host_ptr, 5, N * dmax)
    tables[("host", 4)], tables[("host", 2)] = f32, f16
    tables[("hbm", 4)], tables[("hbm", 2)] = f32.to_device(), f16.to_device()
    hot = np.random.default_rng(3).permutation(N)[: N // 4].astype(np.int64)
    cache = ud.Cache(f32, hot)                                                     # its own launches come before the marker copy
    ids = {"uniform": workloads.indices_uniform(workloads.IDX_STREAM, M, N),
           "stride4": (np.arange(M, dtype=np.int64) * 4) % N,
           "perm": np.random.default_rng(0).permutation(N)[:M].astype(np.int64)}
    ids["sorted"] = np.sort(ids["uniform"])
    dids = {k: torch.from_numpy(v).cuda() for k, v in ids.items()}
    out = torch.empty(max(M * dmax, (2 << 30) // 4), dtype=torch.float32, device="cuda")
    src = torch.empty(M * dmax, dtype=torch.float32, device="cuda").uniform_(-1, 1)
    stream = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()

    # marker and yardstick: a plain copy of exactly 1 GiB (reads 1 GiB, writes 1 GiB)
    bl.udb_plain_copy(out.data_ptr() + (1 << 30), out.data_ptr(), 1 << 30, stream)
    torch.cuda.synchronize()

    rows = []
    for k, (name, kind, dtype, D, where, idkind, tun) in enumerate(replay_shapes(ud)):
        esz = 4 if dtype == ud.UD_F32 else 2
        oesz = 2 if dtype == ud.UD_F16 else 4
        t = tables[(where, esz)]
        view_rows = N if kind != "gather" or idkind != "stride4" else N      # every view has N rows of D elements
        d = dids[idkind]
        ms = []
        for rep in range(REPLAY_LAUNCHES):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            if kind == "gather":
                ud.ud_gather_tuned(t.device_ptr, view_rows, D, dtype, d.data_ptr(), ud.UD_I64, M, out.data_ptr(), stream, tun)
            elif kind == "cached":
                ud.ud_gather_cached(cache.handle, dtype, d.data_ptr(), ud.UD_I64, M, out.data_ptr(), stream)
            else:
                ud.ud_scatter(t.device_ptr, view_rows, D, dtype, d.data_ptr(), ud.UD_I64, M, src.data_ptr(), stream, tun)
            e1.record()
            e1.synchronize()
            ms.append(e0.elapsed_time(e1))
        ud.ud_gather_status(stream)
        plan = None
        if kind == "gather" and tun is None:
            q = ud.ud_gather_plan(t.device_ptr, D, dtype)
            plan = f"lanes={q.lanes_per_row},chunks={q.chunks_per_lane},rows={q.rows_in_flight},max_blocks={q.max_blocks},flags={q.flags}"
        row_in, row_out = D * esz, D * oesz
        if kind == "scatter":
            row_in = row_out = D * esz
        link = where == "host"
        useful = M * (row_in if kind != "scatter" else row_out) if link else M * (row_in + row_out)
        peak = (d2h if kind == "scatter" else h2d) if link else HBM_PEAK_GBPS
        rows.append({"index": k, "name": name, "kind": kind, "table": where, "D": D, "row_bytes_in": row_in, "row_bytes_out": row_out,
                     "launches": REPLAY_LAUNCHES, "ms": round(min(ms[1:]), 4), "useful_bytes": useful,
                     "algorithmic_bytes": M * (row_in + row_out + 8), "peak_GBps": round(peak, 2), "peak_kind": "host link" if link else "HBM",
                     "plan": plan, "rows": M, "mean_128B_lines_per_row": round(_mean_lines_per_row(row_in if kind != "scatter" else row_out), 4)})
        print(f"{k:3d} {name:62s} {min(ms[1:]):9.4f} ms {useful / min(ms[1:]) / 1e6:9.2f} GB/s = {100 * useful / min(ms[1:]) / 1e6 / peak:5.1f}% of the {rows[-1]['peak_kind']} peak",
              flush=True)
    if args.json:
        with open(args.json, "w") as f:
            json.dump({"device": torch.cuda.get_device_name(0), "build_id": ud.ud_build_id(), "h2d_peak_GBps": h2d, "d2h_peak_GBps": d2h,
                       "rows_per_launch": M, "table_rows": N, "shapes": rows}, f)
    cache.free()
    for t in tables.values():
        t.free()
    return 0


def _read_counter_csv(path: str):
    """{counter: [value per dispatch of this library's kernels, in dispatch order, from the marker copy on]},
    and the marker copy's own values."""
    per_dispatch = {}
    names = {}
    for r in csv.DictReader(open(path)):
        d = int(r["Dispatch_Id"])
        names[d] = r["Kernel_Name"]
        per_dispatch.setdefault(d, {})[r["Counter_Name"]] = float(r["Counter_Value"])
    order = sorted(per_dispatch)
    marker = next((d for d in order if "plain_copy_kernel" in names[d]), None)
    if marker is None:
        raise SystemExit(f"{path}: no plain_copy_kernel dispatch (not a --replay run?)")
    ours = [d for d in order if d > marker and any(m in names[d] for m in KERNEL_MARKS)]
    return per_dispatch[marker], [per_dispatch[d] for d in ours], [names[d] for d in ours]


def _summarise(timing_path: str, csv_paths, out_path, traffic_note=None, only=None, note=None) -> int:
    import re
    timing = json.load(open(timing_path))
    shapes = timing["shapes"]
    counters = [{} for _ in shapes]
    kernels = [None] * len(shapes)
    copy_vals = {}
    for path in csv_paths:
        marker, vals, names = _read_counter_csv(path)
        copy_vals.update(marker)
        if len(vals) != sum(s["launches"] for s in shapes):
            raise SystemExit(f"{path}: {len(vals)} kernel dispatches, the timing file expects {sum(s['launches'] for s in shapes)}")
        pos = 0
        for k, s in enumerate(shapes):
            pos += s["launches"]
            counters[k].update(vals[pos - 1])                       # the last launch of the shape
            kernels[k] = names[pos - 1]
    gib_kib = float(1 << 20)
    fscale = gib_kib / copy_vals["FETCH_SIZE"] if copy_vals.get("FETCH_SIZE") else None
    wscale = gib_kib / copy_vals["WRITE_SIZE"] if copy_vals.get("WRITE_SIZE") else None
    lines = []
    w = lines.append
    if note:
        w(f"# {note}")
    w("# made by: python3 -m paper_2101_07956_amd.tune --summarise <timing> <counter files...>, from")
    w("#   python3 -m paper_2101_07956_amd.tune --replay --json <timing>            (plain run: HIP-event times)")
    for path in csv_paths:
        found = sorted({r["Counter_Name"] for r in csv.DictReader(open(path))})
        w(f"#   rocprofv3 --pmc {' '.join(found)} -f csv -d <dir> -o <name> -- python3 -m paper_2101_07956_amd.tune --replay")
    w(f"# Tuning table of the row-gather library on {timing['device']} (build {timing['build_id']}): one row per launch shape.")
    w(f"# {timing['rows_per_launch']:,} rows per launch, tables of {timing['table_rows']:,} rows; HIP-event time of an unprofiled run; peaks of that run:")
    w(f"#   host link {timing['h2d_peak_GBps']:.2f} GB/s (pinned hipMemcpy H2D), {timing['d2h_peak_GBps']:.2f} GB/s (D2H, for the write direction); HBM {HBM_PEAK_GBPS:.0f} GB/s (published)")
    w("# GB/s = useful bytes / time: bytes over the link for host tables, bytes read + written for HBM tables.")
    if fscale:
        w(f"# fetch_MB / write_MB = rocprofv3 FETCH_SIZE / WRITE_SIZE (KiB) scaled by what the same counter reads for the plain 1 GiB copy")
        w(f"#   kernel the replay starts with: FETCH_SIZE x {fscale:.4f}" + (f", WRITE_SIZE x {wscale:.4f}" if wscale else ""))
    w("# floor_MB = rows x (mean number of 128-byte lines a row of the dense layout overlaps) x 128 + the ID list: what a kernel that fetches")
    w("#   every line once must read; traffic/alg = (fetch + write) / algorithmic bytes (row in + row out + 8-byte ID).")
    w("# req128/row = TCC_EA0_RDREQ_128B per gathered row; stalls = TCC_EA0_RDREQ_{IO,DRAM}_CREDIT_STALL (cycles summed over channels).")
    w("")
    hdr = f"{'shape':64s} {'ms':>9s} {'GB/s':>9s} {'%peak':>6s} {'peak':>9s}"
    if fscale:
        hdr += f" {'fetch_MB':>9s} {'floor_MB':>9s} {'fetch/floor':>11s}"
    if wscale:
        hdr += f" {'write_MB':>9s} {'useful_w_MB':>11s}"
    if fscale and wscale:
        hdr += f" {'traffic/alg':>11s}"
    have = set().union(*[set(c) for c in counters]) if counters else set()
    if "TCC_EA0_RDREQ_128B_sum" in have:
        hdr += f" {'req128/row':>10s}"
    for cname, label in (("TCC_EA0_RDREQ_IO_CREDIT_STALL_sum", "IO_stall"), ("TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum", "DRAM_stall")):
        if cname in have:
            hdr += f" {label:>12s}"
    other = sorted(c for c in have if c not in ("FETCH_SIZE", "WRITE_SIZE", "TCC_EA0_RDREQ_128B_sum", "TCC_EA0_RDREQ_IO_CREDIT_STALL_sum",
                                                "TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum"))
    for c in other:
        hdr += f" {c.replace('_sum', ''):>22s}"
    w(hdr)
    for s, c, kn in zip(shapes, counters, kernels):
        if only and not re.search(only, s["name"]):
            continue
        gbps = s["useful_bytes"] / s["ms"] / 1e6
        line = f"{s['name']:64s} {s['ms']:9.4f} {gbps:9.2f} {100 * gbps / s['peak_GBps']:6.1f} {s['peak_kind']:>9s}"
        read_row = s["row_bytes_in"] if s["kind"] != "scatter" else s["row_bytes_out"]
        floor = s["rows"] * (s["mean_128B_lines_per_row"] * 128 + 8) if s["kind"] != "scatter" else s["rows"] * (read_row + 8)
        if fscale:
            f = c.get("FETCH_SIZE")
            line += (f" {f * fscale * 1024 / 1e6:9.1f} {floor / 1e6:9.1f} {f * fscale * 1024 / floor:11.3f}" if f is not None else " " * 31)
        if wscale:
            wv = c.get("WRITE_SIZE")
            line += (f" {wv * wscale * 1024 / 1e6:9.1f} {s['rows'] * s['row_bytes_out'] / 1e6:11.1f}" if wv is not None else " " * 21)
        if fscale and wscale and c.get("FETCH_SIZE") is not None and c.get("WRITE_SIZE") is not None:
            line += f" {(c['FETCH_SIZE'] * fscale + c['WRITE_SIZE'] * wscale) * 1024 / s['algorithmic_bytes']:11.3f}"
        elif fscale and wscale:
            line += " " * 12
        if "TCC_EA0_RDREQ_128B_sum" in have:
            line += f" {c.get('TCC_EA0_RDREQ_128B_sum', float('nan')) / s['rows']:10.3f}"
        for cname in ("TCC_EA0_RDREQ_IO_CREDIT_STALL_sum", "TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum"):
            if cname in have:
                line += f" {c.get(cname, float('nan')):12.0f}"
        for cn in other:
            line += f" {c.get(cn, float('nan')):22.0f}"
        w(line)
    w("")
    w("# kernel of each shape (as the profiler names it):")
    for s, kn in zip(shapes, kernels):
        if kn and not (only and not re.search(only, s["name"])):
            w(f"#   {s['name']:64s} {kn.replace('void ud::', '').replace('(ud::GatherArgs, int)', '').replace('(ud::GatherArgs, ud::FlatArgs)', '').replace('(ud::GatherArgs)', '')}")
    if traffic_note and fscale and wscale:
        # what bench.py prints as roofline.traffic: the D=602 gathers' measured fabric traffic, with the launch shape
        # it belongs to, so that the benchmark can tell when the library has moved on from it
        by_name = {s["name"]: (s, c) for s, c in zip(shapes, counters)}
        host, hbm = by_name.get("gather host f32 D=602 auto"), by_name.get("gather hbm f32 D=602 auto")
        with open(traffic_note, "w") as f:
            f.write("# Fabric traffic per launch of the D=602 fp32 gathers (1,000,000 rows, int64 IDs), from the tuning table's counter runs\n"
                    "# (python3 -m paper_2101_07956_amd.tune --replay under rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE; see gather_tuning_table.txt).\n"
                    f"# build {timing['build_id']}; FETCH_SIZE x {fscale:.4f}, WRITE_SIZE x {wscale:.4f} (scaled by the plain 1 GiB copy kernel)\n")
            for key, pkey, entry in (("", "plan", host), ("hbm_variant_", "hbm_plan", hbm)):
                if not entry or entry[1].get("FETCH_SIZE") is None or entry[1].get("WRITE_SIZE") is None:
                    continue
                sh, c = entry
                fb, wb = c["FETCH_SIZE"] * fscale * 1024, c["WRITE_SIZE"] * wscale * 1024
                f.write(f"{pkey}={sh['plan']}\n{key}fetch_bytes_per_launch={fb:.0f}\n{key}write_bytes_per_launch={wb:.0f}\n"
                        f"{key}traffic_bytes_per_launch={fb + wb:.0f}\n{key}algorithmic_bytes_per_launch={sh['algorithmic_bytes']}\n")
    text = "\n".join(lines) + "\n"
    if out_path:
        with open(out_path, "w") as f:
            f.write(text)
    else:
        sys.stdout.write(text)
    return 0


def _short(name: str) -> str:
    for junk in ("void ud::", "(ud::GatherArgs, int)", "(ud::GatherArgs, ud::FlatArgs)", "(ud::GatherArgs)", "(anonymous namespace)::"):
        name = name.replace(junk, "")
    return name


def _kernel_stats(paths, out_path, note=None) -> int:
    """rocprofv3's *_kernel_stats.csv (and, if given, *_kernel_trace.csv) as a short text table."""
    lines = ([f"# {note}"] if note else []) + [
        "# made by: python3 -m paper_2101_07956_amd.tune --kernel-stats <..._kernel_stats.csv> <..._kernel_trace.csv>", "",
        f"{'kernel':78s} {'calls':>6s} {'avg_ms':>10s} {'min_ms':>10s} {'max_ms':>10s} {'pct':>6s}"]
    for r in csv.DictReader(open(paths[0])):
        n = _short(r["Name"])
        lines.append(f"{n[:78]:78s} {r['Calls']:>6s} {float(r['AverageNs']) / 1e6:10.4f} {float(r['MinNs']) / 1e6:10.4f} "
                     f"{float(r['MaxNs']) / 1e6:10.4f} {float(r['Percentage']):6.2f}")
    if len(paths) > 1:
        agg = {}
        for r in csv.DictReader(open(paths[1])):
            if any(m in r["Kernel_Name"] for m in KERNEL_MARKS):
                grid = r.get("Grid_Size_X") or r.get("Grid_Size")
                agg.setdefault((_short(r["Kernel_Name"]), grid), []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6)
        lines += ["", "# per (kernel, grid size in threads): launches of one width share a grid size"]
        for (k, g), v in agg.items():
            lines.append(f"{k:58s} grid {g:>10s}  calls {len(v):4d}  avg_ms {sum(v) / len(v):9.4f}  min_ms {min(v):9.4f}")
    text = "\n".join(lines) + "\n"
    if out_path:
        with open(out_path, "w") as f:
            f.write(text)
    else:
        sys.stdout.write(text)
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
    ap.add_argument("--replay", action="store_true", help="launch the fixed list of shapes a few times each (for counter runs)")
    ap.add_argument("--summarise", nargs="+", default=None, metavar="FILE",
                    help="replay timing JSON followed by rocprofv3 counter_collection.csv files: print the merged table")
    ap.add_argument("--out", default=None, help="with --summarise: write the table here instead of stdout")
    ap.add_argument("--kernel-stats", nargs="+", default=None, metavar="CSV",
                    help="rocprofv3 *_kernel_stats.csv [and *_kernel_trace.csv]: print them as a short table")
    ap.add_argument("--only", default=None, metavar="REGEX", help="with --summarise: keep the shapes whose name matches")
    ap.add_argument("--note", default=None, help="with --summarise / --kernel-stats: first line of the output")
    ap.add_argument("--traffic-note", default=None, metavar="FILE",
                    help="with --summarise (FETCH_SIZE and WRITE_SIZE files given): also write the D=602 traffic figures bench.py reports")
    args = ap.parse_args()
    if args.amplification:
        return _amplification(args.amplification, args.scale)
    if args.kernel_stats:
        return _kernel_stats(args.kernel_stats, args.out, args.note)
    if args.summarise:
        return _summarise(args.summarise[0], args.summarise[1:], args.out, args.traffic_note, args.only, args.note)
    if args.replay:
        return _replay(args)

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
        # launches back to back between one pair of events: sub-millisecond kernels measured one at a time,
        # with a host round trip between them, read several percent low
        ud.ud_gather_tuned(tptr, N, D, ud.UD_F32, idx.data_ptr(), ud.UD_I64, M, out.data_ptr(), stream, tun)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.reps):
            ud.ud_gather_tuned(tptr, N, D, ud.UD_F32, idx.data_ptr(), ud.UD_I64, M, out.data_ptr(), stream, tun)
        e1.record()
        e1.synchronize()
        return useful / (e0.elapsed_time(e1) / args.reps) / 1e6

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
            if where == "hbm":
                for p in (1, 2, 4):
                    for flags in (ud.UD_TUNE_DEST_ALIGNED, ud.UD_TUNE_DEST_ALIGNED | ud.UD_TUNE_NT_STORE):
                        g = rate(tptr, D, ud.ud_tuning(0, p, 0, 0, flags), useful)
                        res.append({"GBps": round(g, 2), "lanes": 0, "rows_in_flight": 0, "chunks_per_lane": p, "max_blocks": 0,
                                    "flags": flags})
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
