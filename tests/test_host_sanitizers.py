"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the C oracle and the C++ scheduler are
compiled with -fsanitize=address,undefined together with a driver that takes every entry point through
small ragged problems with exact-size heap buffers (tests/sanitize/), and the drivers must run clean.
(GPU code cannot be run under a sanitizer here; its bounds are covered by guard rows, poisoned padding
and ALISE_DEBUG_VALIDATE in the GPU tests.)"""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan"]


def _build_and_run(tmp_path, compiler, std, sources, extra=()):
    exe = str(tmp_path / "driver")
    cmd = [compiler, std, *SAN, *extra, "-o", exe, *[os.path.join(ROOT, s) for s in sources], "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and ("asan" in built.stderr or "ubsan" in built.stderr) and "error:" not in built.stderr:
        pytest.skip("the sanitizer runtimes are not installed for this compiler")
    assert built.returncode == 0, built.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-3000:]
    return run.stdout


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    out = _build_and_run(tmp_path, "gcc", "-std=c11", ["tests/sanitize/oracle_driver.c", "oracle/alise_oracle.c"],
                         extra=("-ffp-contract=off", "-fopenmp"))
    assert "ok" in out


def test_scheduler_runs_clean_under_asan_and_ubsan(tmp_path):
    out = _build_and_run(tmp_path, "g++", "-std=c++17", ["tests/sanitize/sched_driver.cpp", "paper_2410_23537_amd/csrc/sched.cpp"])
    assert "ok" in out
