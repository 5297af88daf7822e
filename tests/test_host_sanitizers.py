"""The host-side scheduler under AddressSanitizer + UBSan (g++, no GPU): random sessions against a
back end that checks the consistency of every launch."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_scheduler_fuzz_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_fuzz")
    src = os.path.join(HERE, "native", "host_fuzz.cpp")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-Wall", "-Wextra", src, "-o", exe], check=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=1:verify_asan_link_order=0"
    res = subprocess.run([exe, "2500"], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.startswith("ok 2500 sessions")
