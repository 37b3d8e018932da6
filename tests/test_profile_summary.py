"""profile_summary.py on small hand-made files in rocprofv3's CSV layout: kernel names are told
apart by their template arguments, counter readings are calibrated by the plain copy, and the
traffic ratio comes out as bytes moved over bytes the table asks for.  CPU only."""
import csv
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NS = "void mempool::(anonymous namespace)::"
TAIL = "(mempool::(anonymous namespace)::CopyArgs, int const*, int const*)"
HEAD = ["Correlation_Id", "Dispatch_Id", "Agent_Id", "Queue_Id", "Process_Id", "Thread_Id", "Grid_Size", "Kernel_Id",
        "Kernel_Name", "Workgroup_Size", "LDS_Block_Size", "Scratch_Size", "VGPR_Count", "Accum_VGPR_Count",
        "SGPR_Count", "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"]


def _counter_file(path, counter, rows):
    os.makedirs(path, exist_ok=True)
    with open(os.path.join(path, "bench_counter_collection.csv"), "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(HEAD)
        for i, (name, grid, value) in enumerate(rows):
            w.writerow([i, i, "Agent 1", 1, 1, 1, grid, 1, name, 64, 0, 0, 8, 0, 16, counter, value, 0, 1])


def test_traffic_and_stats_summaries(tmp_path):
    sys.path.insert(0, ROOT)
    import profile_summary as P
    assert P.short(NS + "kv_block_copy<1, true, 1, 0>" + TAIL) == "kv_block_copy<1,true,1> gather"
    assert P.short(NS + "kv_block_copy<2, false, 4, 2>" + TAIL) == "kv_block_copy<2,false,4> fused"
    assert P.short(NS + "plain_copy_kernel(HIP_vector_type<unsigned int, 4u> const*)") == "plain_copy_kernel"
    assert P.short("void at::native::vectorized_elementwise_kernel<4>(int)") is None
    # plain copy: 65536 threads x 16 B = 1024 KiB each way; FETCH_SIZE counts 2 KiB units, WRITE_SIZE 1 KiB
    plain = NS + "plain_copy_kernel(unsigned int const*, unsigned int*, unsigned long)"
    gather = NS + "kv_block_copy<1, true, 1, 0>" + TAIL
    scatter = NS + "kv_block_copy<1, true, 1, 1>" + TAIL
    grid = 64 * 2048                                   # 2048 wave-items of 1 KiB
    _counter_file(str(tmp_path / "fetch"), "FETCH_SIZE", [(plain, 65536, 512.0), (gather, grid, 1024.0), (scatter, grid, 1126.4)])
    _counter_file(str(tmp_path / "write"), "WRITE_SIZE", [(plain, 65536, 1024.0), (gather, grid, 2048.0), (scatter, grid, 2048.0)])
    out, js = str(tmp_path / "t.txt"), str(tmp_path / "t.json")
    subprocess.check_call([sys.executable, os.path.join(ROOT, "profile_summary.py"), "traffic", str(tmp_path / "fetch"),
                           str(tmp_path / "write"), "--out", out, "--json", js, "--cmd", "test"], stdout=subprocess.DEVNULL)
    j = json.load(open(js))
    assert j["fetch_scale_KiB_per_count"] == 2.0 and j["write_scale_KiB_per_count"] == 1.0
    assert j["traffic_per_algorithmic_byte"]["gather"] == 1.0            # 2048 KiB read + 2048 KiB written
    assert j["traffic_per_algorithmic_byte"]["scatter"] == 1.05          # 10 % of the reads fetched twice
    assert j["kernel_source_sha"] == P.kernel_sha()
    assert "kv_block_copy<1,true,1> scatter" in open(out).read()
    # kernel statistics
    os.makedirs(tmp_path / "stats")
    with open(tmp_path / "stats" / "bench_kernel_stats.csv", "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"])
        w.writerow([gather, 4, 4000, 1000.0, 40.0, 900, 1100, 1.0])
        w.writerow(["void at::native::fill_kernel(int)", 9, 9000, 1000.0, 60.0, 900, 1100, 1.0])
    out2 = str(tmp_path / "s.txt")
    subprocess.check_call([sys.executable, os.path.join(ROOT, "profile_summary.py"), "stats", str(tmp_path / "stats"),
                           "--out", out2, "--cmd", "test"], stdout=subprocess.DEVNULL)
    text = open(out2).read()
    assert "kv_block_copy<1,true,1> gather" in text and "fill_kernel" not in text
