"""The host planner and the per-pair host arithmetic under the address and undefined-behaviour
sanitizers: tests/planner_fuzz.cpp feeds them seeded random row-pointer arrays, options and rows
(no GPU, no oracle: what is checked is that nothing reads or writes out of bounds, nothing
overflows, and every plan that is made passes the planner's own consistency check)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_and_pair_arithmetic_under_sanitizers(tmp_path):
    exe = str(tmp_path / "planner_fuzz")
    csrc = os.path.join(ROOT, "paper_2104_06357_amd", "csrc")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-I" + os.path.join(ROOT, "include"), "-I" + csrc,
           os.path.join(ROOT, "tests", "planner_fuzz.cpp"), os.path.join(csrc, "spd_plan.cpp"),
           os.path.join(csrc, "spd_testing.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "sanitize" in build.stderr and "cannot find" in build.stderr:
        pytest.skip("the sanitizer runtimes are not installed")
    assert build.returncode == 0, build.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe, "1500"], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    last = run.stdout.strip().splitlines()[-1].split()
    assert last[0] == "planned" and int(last[1]) > 1000 and last[4] == "inconsistent" and int(last[5]) == 0, run.stdout[-500:]
