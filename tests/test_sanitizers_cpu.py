"""The CPU oracle and the library's host-only code (chunk scheduler) built with
AddressSanitizer and UndefinedBehaviorSanitizer and run on shapes that reach every
loop tail.  GPU code cannot be sanitized on this machine; this covers what runs on the
host."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_scheduler_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-static-libubsan", "-Wall", "-Wextra",
           "-I", os.path.join(ROOT, "paper_2410_10989_amd", "csrc"),
           os.path.join(ROOT, "oracle", "flce_oracle.cpp"),
           os.path.join(ROOT, "tests", "oracle_sanitize_main.cpp"), "-o", exe]
    b = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert b.returncode == 0, b.stdout
    env = dict(os.environ, OMP_NUM_THREADS="4",
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env,
                       timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "all checks passed" in r.stdout
    assert "AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout
