"""The host-only part of the library (table rules, tile planning, write-set runs, replication,
timing statistics) built with AddressSanitizer and UndefinedBehaviorSanitizer and driven by
tests/host_sanitized_main.cpp on the CPU.  No GPU code is involved: the two files compiled here
use the HIP headers only for type names."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_sanitized")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"),
           "-I" + os.path.join(ROOT, "paper_2604_11109_amd", "csrc"),
           os.path.join(ROOT, "tests", "host_sanitized_main.cpp"),
           os.path.join(ROOT, "paper_2604_11109_amd", "csrc", "r3_table.cpp"), "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert built.returncode == 0, built.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    ran = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert ran.returncode == 0, (ran.stdout[-2000:], ran.stderr[-4000:])
    assert "host checks passed" in ran.stdout
