"""The host-side (integer) part of the library and the CPU oracle under AddressSanitizer and
UndefinedBehaviorSanitizer.  CPU only: sanitizers run on host code, never on the GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_and_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2602_15563_amd", "csrc"),
           os.path.join(ROOT, "tests", "native", "host_sanitize_main.cpp"),
           os.path.join(ROOT, "paper_2602_15563_amd", "csrc", "kmq_host.cpp"),
           os.path.join(ROOT, "oracle", "kmq_oracle.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    # another preloaded library may come before the sanitizer runtime in the link order
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host sanitizer run: ok" in r.stdout
