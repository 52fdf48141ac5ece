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
