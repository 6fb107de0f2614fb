"""The library's host code and the CPU checker under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_and_checker_run_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    csrc = os.path.join(ROOT, "paper_2206_10620_amd", "csrc")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-static-libasan", "-static-libubsan",      # the runtimes inside the executable: no demand on the order of preloaded libraries
           "-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(ROOT, "tests", "host_sanitize_main.cpp"), os.path.join(csrc, "plan.cpp"), os.path.join(csrc, "block_plan.cpp"),
           os.path.join(ROOT, "oracle", "pp_oracle.cpp"), os.path.join(ROOT, "oracle", "pp_block_oracle.cpp"),
           os.path.join(ROOT, "oracle", "pp_reuse_oracle.cpp"), "-pthread", "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-6000:])
    assert r.stdout.startswith("ok ")
