"""The host half of the library (argument validation, tiling plans, workspace layout: ea_host.cpp)
built with AddressSanitizer and UndefinedBehaviorSanitizer and driven over a sweep of shapes by
tests/native/host_sanitize_main.cpp.  CPU only; the GPU code is not built with sanitizers."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_host_code_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_san")
    cmd = ["g++", "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-o", exe, os.path.join(ROOT, "tests", "native", "host_sanitize_main.cpp"),
           os.path.join(ROOT, "paper_2510_00636_amd", "csrc", "ea_host.cpp")]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host checks passed" in r.stdout
