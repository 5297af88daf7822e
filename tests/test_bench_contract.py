"""The parts of bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_measured_traffic_is_tied_to_the_kernel_configuration_string():
    # counter figures are only reported while the library says it was built with the launch shapes the
    # counters were taken with; whatever is recorded must be close to the bytes the launches are known to move
    sys.path.insert(0, ROOT)
    import bench
    import paper_2002_05814_amd as hop
    assert bench.profiled_traffic("cfg2_async_sgd", "some other shape") is None
    if bench.PROFILED_TRAFFIC["workloads"]:
        assert bench.PROFILED_TRAFFIC["kernel_config"] == hop.hop_kernel_config()
    moved = {"cfg2_async_sgd": 13 * 64 << 20, "cfg3_rl_allreduce": (65 + 64) * 16 << 20,
             "cfg4_large_fault": (10 * (33 + 6) + 10 * (6 + 5 + 1) + 22 * 32) * 8 << 20,
             "cfg4_large_fault_without_failure": 33 * 256 << 20}
    for name, entry in bench.PROFILED_TRAFFIC["workloads"].items():
        assert os.path.exists(os.path.join(ROOT, entry["profile"]))
        if name in moved:
            assert abs(entry["bytes_per_call"] - moved[name]) / moved[name] < 0.02, name
