"""The counter-file summariser of the tuning tool (no GPU): bytes per launch from a rocprofv3 --pmc CSV."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CSV = '''"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id","Kernel_Name","Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count","Counter_Name","Counter_Value","Start_Timestamp","End_Timestamp"
1,1,"Agent 1",1,1,1,2097152,1,"(anonymous namespace)::plain_copy_kernel(HIP_vector_type<unsigned int, 4u> const*, HIP_vector_type<unsigned int, 4u>*, unsigned long)",256,0,0,8,0,32,"FETCH_SIZE",524288.0,1,2
2,2,"Agent 1",1,1,1,131072,2,"void ud::gather_chunked<0, 1, 3, false, false>(ud::GatherArgs, int)",256,0,0,48,0,32,"FETCH_SIZE",1250000.0,3,4
3,3,"Agent 1",1,1,1,131072,2,"void ud::gather_chunked<0, 1, 3, false, false>(ud::GatherArgs, int)",256,0,0,48,0,32,"FETCH_SIZE",1250000.0,5,6
'''


def test_amplification_summary(tmp_path):
    f = tmp_path / "fetch_counter_collection.csv"
    f.write_text(CSV)
    r = subprocess.run([sys.executable, "-m", "paper_2101_07956_amd.tune", "--amplification", str(f), "--scale", "2.0"],
                       capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 0, r.stderr
    assert "scale 2.0000" in r.stdout                                   # 1 GiB copy read as 524288 KiB
    line = [l for l in r.stdout.splitlines() if "gather_chunked<0, 1, 3" in l][0]
    assert line.split()[-1] == "2560.0" and " 2 " in line               # 1,250,000 KiB x 2 = 2560 MB, two launches


def _row(disp, kernel, counter, value):
    return (f'{disp},{disp},"Agent 1",1,1,1,1024,1,"{kernel}",256,0,0,8,0,32,"{counter}",{value},1,2\n')


def test_replay_counter_files_merge_into_one_table(tmp_path):
    # two shapes, three launches each; a FETCH_SIZE file and a WRITE_SIZE + request-count file from separate runs
    import json
    timing = {"device": "test", "build_id": "x", "h2d_peak_GBps": 50.0, "d2h_peak_GBps": 50.0, "rows_per_launch": 1000, "table_rows": 4000,
              "shapes": [{"index": 0, "name": "gather host f32 D=32 auto", "kind": "gather", "table": "host", "D": 32, "row_bytes_in": 128,
                          "row_bytes_out": 128, "launches": 3, "ms": 0.004, "useful_bytes": 128000, "algorithmic_bytes": 264000,
                          "peak_GBps": 50.0, "peak_kind": "host link", "rows": 1000, "mean_128B_lines_per_row": 1.0},
                         {"index": 1, "name": "gather hbm f32 D=602 auto", "kind": "gather", "table": "hbm", "D": 602, "row_bytes_in": 2408,
                          "row_bytes_out": 2408, "launches": 3, "ms": 0.001, "useful_bytes": 4816000, "algorithmic_bytes": 4824000,
                          "peak_GBps": 8000.0, "peak_kind": "HBM", "rows": 1000, "mean_128B_lines_per_row": 19.75}]}
    (tmp_path / "timing.json").write_text(json.dumps(timing))
    hdr = CSV.splitlines()[0] + "\n"
    copy = "(anonymous namespace)::plain_copy_kernel(x)"
    g1, g2 = "void ud::gather_chunked<0, 1, 1, false, true>(ud::GatherArgs, int)", "void ud::gather_flat<0, 2, true, true>(ud::GatherArgs, ud::FlatArgs)"
    fetch = hdr + _row(1, "void ud::gather_chunked<0, 1, 1, false, true>(ud::GatherArgs, int)", "FETCH_SIZE", 7)   # cache fill: before the marker
    fetch += _row(2, copy, "FETCH_SIZE", 524288.0)
    for d, (k, v) in enumerate([(g1, 1), (g1, 2), (g1, 66.40625), ("fetch_and_reset(x)", 0), (g2, 1), (g2, 2), (g2, 1238.28125)], start=3):
        fetch += _row(d, k, "FETCH_SIZE", v)
    (tmp_path / "fetch.csv").write_text(fetch)
    wr = hdr + _row(1, copy, "WRITE_SIZE", 1048576.0) + _row(1, copy, "TCC_EA0_RDREQ_128B_sum", 8388608)
    for d, (k, v, q) in enumerate([(g1, 0, 0), (g1, 0, 0), (g1, 125.0, 1000), (g2, 0, 0), (g2, 0, 0), (g2, 2351.5625, 19750)], start=2):
        wr += _row(d, k, "WRITE_SIZE", v) + _row(d, k, "TCC_EA0_RDREQ_128B_sum", q)
    (tmp_path / "write.csv").write_text(wr)
    r = subprocess.run([sys.executable, "-m", "paper_2101_07956_amd.tune", "--summarise", str(tmp_path / "timing.json"),
                        str(tmp_path / "fetch.csv"), str(tmp_path / "write.csv")], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 0, r.stderr
    rows = [l for l in r.stdout.splitlines() if l.startswith("gather ")]
    assert len(rows) == 2
    a = rows[0].split()
    # 128,000 useful bytes in 0.004 ms = 32 GB/s = 64% of 50; fetched 66.40625 KiB x 2.0 = 136,000 B = the floor (1000 x (128 + 8))
    assert a[a.index("auto") + 1: a.index("auto") + 4] == ["0.0040", "32.00", "64.0"]
    assert "1.000" in a and "0.1" in a                               # fetch / floor, fetch_MB
    b = rows[1].split()
    assert "19.750" in b                                             # read requests per row
    assert "gather_flat<0, 2, true, true>" in r.stdout               # the kernel behind each shape is named
