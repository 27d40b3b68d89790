"""The CPU oracle built with AddressSanitizer and UndefinedBehaviorSanitizer and driven once over all its routines on
ragged, empty and extreme inputs (tests/oracle_sanitize_driver.cpp): the checker must itself be free of out-of-bounds
accesses and undefined arithmetic before its outputs are used to judge anything."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "oracle_sanitize_driver")
    cmd = [gxx, "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", os.path.join(HERE, "oracle_sanitize_driver.cpp"),
           "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "cannot find" in build.stderr:
        pytest.skip("sanitizer runtimes are not installed: " + build.stderr.strip().splitlines()[-1])
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, run.stderr[-4000:]
    assert "done" in run.stdout and "runtime error" not in run.stderr and "ERROR: AddressSanitizer" not in run.stderr
