"""The rocprofv3-CSV summariser on hand-made traces: per-kernel statistics, the concurrency
histogram of a replay and the scaling of the traffic counters by the calibration kernel."""
import csv
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    p = subprocess.run([sys.executable, "-m", "paper_2312_10351_amd.profile_summary", *args], cwd=ROOT,
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert p.returncode == 0, p.stderr
    return p.stdout


def write_trace(path, rows):
    cols = ["Kind", "Agent_Id", "Queue_Id", "Stream_Id", "Thread_Id", "Dispatch_Id", "Kernel_Id", "Kernel_Name",
            "Correlation_Id", "Start_Timestamp", "End_Timestamp", "LDS_Block_Size", "Scratch_Size", "VGPR_Count",
            "Accum_VGPR_Count", "SGPR_Count", "Workgroup_Size_X", "Workgroup_Size_Y", "Workgroup_Size_Z",
            "Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z"]
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(cols)
        for i, (name, q, t0, t1) in enumerate(rows):
            w.writerow(["KERNEL_DISPATCH", "Agent 1", q, 0, 1, i + 1, 1, name, i + 1, t0, t1, 0, 0, 8, 0, 16, 256, 1, 1, 512, 1, 1])


def write_counter(path, counter, rows):
    cols = ["Correlation_Id", "Dispatch_Id", "Agent_Id", "Queue_Id", "Process_Id", "Thread_Id", "Grid_Size", "Kernel_Id",
            "Kernel_Name", "Workgroup_Size", "LDS_Block_Size", "Scratch_Size", "VGPR_Count", "Accum_VGPR_Count", "SGPR_Count",
            "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"]
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(cols)
        for i, (name, v) in enumerate(rows):
            w.writerow([i + 1, i + 1, "Agent 1", 1, 1, 1, 512, 1, name, 256, 0, 0, 8, 0, 16, counter, float(v), 0, 1])


def test_stats_and_overlap(tmp_path):
    d = tmp_path / "trace"
    d.mkdir()
    # two replays of three kernels: a runs 0-10, b 5-15 (overlaps a for 5), c 20-30
    rows = []
    for base in (0, 100000):
        rows += [("opara_k_a", 1, base + 0, base + 10000), ("opara_k_b", 2, base + 5000, base + 15000),
                 ("opara_k_c", 1, base + 20000, base + 30000)]
    rows.append(("other_kernel", 1, 5, 6))
    write_trace(d / "t_kernel_trace.csv", rows)
    out = run("stats", str(d))
    assert "| opara_k_a | 2 | 10000 | 10000 | 10000 |" in out
    out = run("overlap", str(d), "--kernels", "3", "--replay", "-1", "--timeline", "3")
    assert "3 kernels, span 30.0 us, sum of kernel durations 30.0 us, hardware queues used 2, peak concurrency 2" in out
    assert "| 2 | 16.7 % | 5.0 |" in out and "| 0 | 16.7 % | 5.0 |" in out and "| 1 | 66.7 % | 20.0 |" in out
    assert "mean kernels in flight over the span: 1.00" in out
    assert "| 5.00 | 10.00 | 2 | b | 2 |" in out


def test_traffic_is_scaled_by_the_calibration_kernel(tmp_path):
    f, w = tmp_path / "f", tmp_path / "w"
    f.mkdir(); w.mkdir()
    # the calibration kernel reads and writes 1000 KiB; the fetch counter reads half of it, the write counter all
    write_counter(f / "f_counter_collection.csv", "FETCH_SIZE", [("opara_k_elt_f16_vec", 500), ("opara_k_x", 100), ("opara_k_x", 300)])
    write_counter(w / "w_counter_collection.csv", "WRITE_SIZE", [("opara_k_elt_f16_vec", 1000), ("opara_k_x", 50), ("opara_k_x", 50)])
    target = tmp_path / "traffic.txt"
    out = run("traffic", str(f), str(w), "--workload", "wl", "--calibration-kib", "1000", "--append", str(target))
    assert "fetch x 2.000, write x 1.000" in out
    assert "| opara_k_x | 2 | 200.0 | 50.0 | 400 + 50 = 450 KiB" in out
    lines = dict(l.split()[1:2] + [l.split()[2:]] for l in open(target))
    assert lines["x"] == ["409600", "51200"]
