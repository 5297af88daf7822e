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
    # the counter figure is only reported while the library says it was built with the launch shapes
    # the counters were taken with
    sys.path.insert(0, ROOT)
    import bench
    import paper_2002_05814_amd as hop
    assert bench.MEASURED_TRAFFIC["kernel_config"] == hop.hop_kernel_config()
    algorithmic = 13 * 64 * (1 << 20)
    assert abs(bench.MEASURED_TRAFFIC["bytes"] - algorithmic) / algorithmic < 0.01
