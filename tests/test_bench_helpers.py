"""Host-side helpers of bench.py (no GPU): the traffic figure of the roofline object is read from the tracked
counter summary and is given only for the kernel sources the counters were taken on."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_traffic_line_of_the_tracked_summary_parses():
    lines = [l for l in open(bench.TRAFFIC_PROFILE) if l.startswith("bench_roofline_traffic ")]
    assert len(lines) == 1
    kv = dict(t.split("=", 1) for t in lines[0].split()[1:])
    assert kv["workload"] == "cfg3" and kv["family"] == "gemm_tn" and len(kv["kernel_sources_sha256"]) == 64
    # algorithmic bytes of one weight-gradient GEMM call are 0.59 GB; the counters must be above that and below 4x
    assert 0.59e9 < float(kv["bytes_per_launch"]) < 2.4e9


def test_traffic_is_given_only_for_the_recorded_kernel_sources(monkeypatch):
    kv = dict(t.split("=", 1) for l in open(bench.TRAFFIC_PROFILE) if l.startswith("bench_roofline_traffic ") for t in l.split()[1:])
    monkeypatch.setattr(bench, "kernel_sources_sha256", lambda: kv["kernel_sources_sha256"])
    assert bench.measured_traffic("cfg3", "gemm_tn") == float(kv["bytes_per_launch"])
    assert bench.measured_traffic("cfg2", "gemm_tn") is None and bench.measured_traffic("cfg3", "gemm_nt") is None
    monkeypatch.setattr(bench, "kernel_sources_sha256", lambda: "0" * 64)
    assert bench.measured_traffic("cfg3", "gemm_tn") is None


def test_more_than_one_gpu_is_refused():
    import subprocess
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
