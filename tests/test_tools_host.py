"""Host-side checks of the measurement tooling (no GPU): bench.py refuses more than one GPU and says why, and
paper_2604_24088_amd.profile_summary turns rocprofv3-shaped CSV files and bench lines into the tables kept under
profiles/ (synthetic files with known values in, the derived figures out)."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(args, **kw):
    return subprocess.run([sys.executable] + args, cwd=ROOT, capture_output=True, text=True, timeout=120, **kw)


def test_bench_refuses_more_than_one_gpu():
    r = run(["bench.py", "--gpus", "2"])
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr
    env = dict(os.environ, WORLD_SIZE="4")
    r = run(["bench.py"], env=env)
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def write_csv(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write(",".join(header) + "\n")
        for row in rows:
            f.write(",".join(f'"{c}"' if isinstance(c, str) and "," in c else str(c) for c in row) + "\n")


def test_profile_summary_tables(tmp_path):
    from paper_2604_24088_amd import profile_summary as ps

    stats = tmp_path / "stats"
    write_csv(str(stats / "bench_kernel_stats.csv"), ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"],
              [["void taco::compress_mfma_kernel<1, 1, false, 0, false>(taco::CompressTable, int, float, float, int)", 10, 940000, 94000.0, 75.0,
                92000, 97000, 1.0],
               ["taco::copy_kernel(void const*, void*, long)", 2, 300000, 150000.0, 25.0, 149000, 151000, 1.0]])
    rows = ps.kernel_stats(str(stats))
    assert rows[0][0] == "compress_mfma_kernel<1, 1, false, 0, false>" and rows[0][1] == 10 and rows[0][2] == 94000.0
    assert rows[1][0] == "copy_kernel"

    # counters: the copy kernel calibrates the scale (FETCH_SIZE reads half of the 393216 KiB the copy moves)
    fetch = tmp_path / "FETCH_SIZE"
    header = ["Correlation_Id", "Dispatch_Id", "Agent_Id", "Queue_Id", "Process_Id", "Thread_Id", "Grid_Size", "Kernel_Id", "Kernel_Name",
              "Workgroup_Size", "LDS_Block_Size", "Scratch_Size", "VGPR_Count", "Accum_VGPR_Count", "SGPR_Count", "Counter_Name",
              "Counter_Value", "Start_Timestamp", "End_Timestamp"]

    def counter_row(i, grid, name, counter, value):
        return [i, i, 0, 0, 1, 1, grid, 1, name, 64, 0, 0, 64, 0, 32, counter, value, 0, 1]

    write_csv(str(fetch / "bench_counter_collection.csv"), header,
              [counter_row(1, 100, "taco::copy_kernel(void const*, void*, long)", "FETCH_SIZE", 196608.0),
               counter_row(2, 6291456, "void taco::compress_mfma_kernel<1, 1, false, 0, false>(taco::CompressTable, int, float, float, int)",
                           "FETCH_SIZE", 100000.0),
               counter_row(3, 6291456, "void taco::compress_mfma_kernel<1, 1, false, 0, false>(taco::CompressTable, int, float, float, int)",
                           "FETCH_SIZE", 102000.0)])
    tab = ps.counters(str(fetch))
    n, mean = tab[("compress_mfma_kernel<1, 1, false, 0, false>", "6291456", "FETCH_SIZE")]
    assert n == 2 and mean == 101000.0
    assert tab[("copy_kernel", "100", "FETCH_SIZE")] == (1, 196608.0)
    r = run(["-m", "paper_2604_24088_amd.profile_summary", "--fetch", str(fetch)])
    assert r.returncode == 0, r.stderr
    assert "x 2.000000" in r.stdout                      # 393216 / 196608
    assert "scaled=    202000.0 KiB" in r.stdout

    # kernel trace: a launch after another kernel with an idle gap, launches after the same kernel without
    trace_header = ["Kind", "Agent_Id", "Queue_Id", "Stream_Id", "Thread_Id", "Dispatch_Id", "Kernel_Id", "Kernel_Name", "Correlation_Id",
                    "Start_Timestamp", "End_Timestamp"]
    rows, t = [], 0
    for i in range(6):
        rows.append(["KERNEL_DISPATCH", 0, 0, 0, 1, 2 * i, 1, "taco::A(int)", 2 * i, t, t + 1000])
        rows.append(["KERNEL_DISPATCH", 0, 0, 0, 1, 2 * i + 1, 2, "taco::B(int)", 2 * i + 1, t + 1000 + 5000, t + 1000 + 5000 + 3000])
        t += 1000 + 5000 + 3000
    write_csv(str(stats / "bench_kernel_trace.csv"), trace_header, rows)
    r = run(["-m", "paper_2604_24088_amd.profile_summary", "--trace", str(stats)])
    assert r.returncode == 0, r.stderr
    line_b = [ln for ln in r.stdout.splitlines() if ln.strip().startswith("B ")][0]
    assert "duration=     3000" in line_b and "their median gap    5000" in line_b
    line_a = [ln for ln in r.stdout.splitlines() if ln.strip().startswith("A ")][0]
    assert "launches with a gap over 1 us:    0" in line_a

    # bench lines
    call = {"ms": 0.1, "moved_GBps": 6000.0, "hbm_frac": 0.75}
    bench = {"config": {"workload": "large_k8: x", "block": 128, "layout": "split", "impl": "auto", "format": "e4m3", "mode": 7},
             "ms_per_step": 1.2, "hbm_frac_step": 0.8, "calls": {"compress": call, "decompress": call, "decompress_sum_k8": call},
             "calls_back_to_back": {"compress": call, "decompress": call, "decompress_sum_k8": call},
             "mix_yardstick": {"compress": call, "decompress": call, "decompress_sum_k8": call, "decompress_sum_compress_k8": call}}
    path = tmp_path / "line.json"
    path.write_text("some log line\n" + json.dumps(bench) + "\n")
    r = run(["-m", "paper_2604_24088_amd.profile_summary", "--bench", str(path)])
    assert r.returncode == 0, r.stderr
    assert "large_k8 k=8 B=128 split auto fmt=e4m3 mode=7" in r.stdout and "100.0 0.750" in r.stdout
