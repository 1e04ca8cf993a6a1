"""What can be said of bench.py without a GPU: more than one GPU is refused with
a message, and the recorded traffic is attached only while the kernel source is
the one the record was taken with."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_recorded_traffic_is_bound_to_the_kernel_source():
    sys.path.insert(0, ROOT)
    import bench
    name, workload = "group_sync_cfg3_traffic.txt", "cfg3 W=32 g=8 P=25557032 ld=25557248"
    rec = json.load(open(os.path.join(ROOT, "profiles", name)))
    blob = bench.git_blob_id(os.path.join(ROOT, "paper_2007_03298_amd", "csrc", "group_sync.hip"))
    got = bench.measured_traffic(name, workload)
    if rec["kernel_source_blob"] == blob:
        # 12 B per (worker, column), no wasted traffic
        assert got == rec["hbm_bytes_per_launch"]
        assert abs(got / rec["algorithmic_bytes_per_launch"] - 1.0) < 0.01
    else:
        assert got is None          # a record of another kernel is not this kernel's traffic
    assert bench.measured_traffic(name, "some other workload") is None
    assert bench.measured_traffic("no_such_record.txt", workload) is None
