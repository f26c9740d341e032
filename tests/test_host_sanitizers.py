"""Host C++ of the library (batcher, quad-tree generator, scheduler) under
AddressSanitizer and UndefinedBehaviorSanitizer: a small driver runs random
call sequences, including the error paths."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_23389_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_fuzz")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host_fuzz.cpp"), os.path.join(CSRC, "batcher.cpp"),
           os.path.join(CSRC, "quadtree.cpp"), os.path.join(CSRC, "scheduler.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ)
    # other preloaded libraries may precede the sanitizer runtime: accept that order
    env["ASAN_OPTIONS"] = "detect_leaks=1:verify_asan_link_order=0"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host fuzz ok" in r.stdout
