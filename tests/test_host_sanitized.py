"""The library's host-only entry points (queue schedule, bubble count, noise assignment) compiled with
AddressSanitizer and UndefinedBehaviorSanitizer and driven over small grids and extreme sizes
(tests/host_fuzz.cpp): no overflow, no out-of-bounds access, no exception across the C ABI."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_entry_points_under_sanitizers(tmp_path):
    exe = tmp_path / "host_fuzz"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           os.path.join(ROOT, "tests", "host_fuzz.cpp"),
           os.path.join(ROOT, "paper_2505_21070_amd", "csrc", "schedule.cpp"), "-o", str(exe)]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:allocator_may_return_null=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert r.stdout.strip().startswith("ok "), r.stdout[-500:]
