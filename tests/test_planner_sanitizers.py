"""The host planner under AddressSanitizer and UndefinedBehaviorSanitizer: compiled with
g++ (it is pure host C++), run on small shapes with full validation and on the 7B / 70B
shapes without."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_planner_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "planner_san")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2409_19256_amd", "csrc"),
           os.path.join(ROOT, "paper_2409_19256_amd", "csrc", "planner.cpp"),
           os.path.join(ROOT, "tests", "planner_sanitize_main.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    # the runtime is linked statically and told not to insist on being the first library, so
    # the test does not depend on what else the environment preloads
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.count("ok:") == 8
