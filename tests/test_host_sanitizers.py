"""The pure-host half of the library (planner of Sec. 4.1's bookkeeping, plan blob, scheduler
and staleness counters) built with the host compiler's AddressSanitizer and
UndefinedBehaviorSanitizer and run on seeded ragged batches.  No GPU code is compiled or run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_planner_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "host_sanitize")
    csrc = os.path.join(ROOT, "paper_2605_28396_amd", "csrc")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-Wall", "-Werror",
           "-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(csrc, "host_plan.cpp"), os.path.join(ROOT, "tests", "host_sanitize_main.cpp"),
           "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe, "300"], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert r.stdout.strip() == "ok 300 cases"
    assert "runtime error" not in r.stderr and "Sanitizer" not in r.stderr, r.stderr[-4000:]
