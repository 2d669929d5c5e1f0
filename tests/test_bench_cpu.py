"""Host-side checks of bench.py that need no GPU: the one-GPU rule and the bookkeeping of measured traffic."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_traffic_records_are_tied_to_the_kernel_source():
    import bench
    for (workload, cls), rec in bench.TRAFFIC.items():
        assert os.path.exists(os.path.join(ROOT, rec["kernel_source"])), rec["kernel_source"]
        h = bench.source_hash(rec["kernel_source"], rec.get("sections"))
        assert h is not None, (workload, cls, "a named section is missing from the source")
        got = bench.measured_traffic(workload, cls)
        runs = rec["bytes_per_launch_runs"]
        if h == rec["sha256"]:
            assert got == int(sum(runs) / len(runs)) and bench.traffic_min_max(workload, cls) == [min(runs), max(runs)]
        else:
            assert got is None and bench.traffic_min_max(workload, cls) is None  # kernel changed since the counters were taken
    assert bench.measured_traffic("no such workload", "resnet_fused") is None


def test_the_headline_kernels_counters_are_current():
    """The traffic figure of the default line is reported only while the kernel source is the one it was measured on."""
    import bench
    assert bench.measured_traffic("resnet20_greedy_step_n1024_s40", "resnet_fused") is not None
