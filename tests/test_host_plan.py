"""The pure-host part of libdbsn (arena layout, tile geometry of the persistent kernel, choice of
the register layout, shape checks: csrc/dbsn_plan.h) compiled with g++ under AddressSanitizer and
UndefinedBehaviorSanitizer and run over 2,000 random layer shapes (every weight of every layer counted into its tile), no GPU involved."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_planning_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_plan_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-Wall", "-Wextra", "-Werror",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_1003_0358_amd", "csrc"),
           os.path.join(ROOT, "tests", "host_plan_check.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe, "2000"], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.strip() == "ok 2000", r.stdout + r.stderr
