"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only): the fp64 oracle and the
workload generators are each compiled together with a small driver that walks every one of their
entry points on small inputs, and any sanitizer report fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FLAGS = ["-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]


def _build_and_run(tmp_path, compiler, src, extra):
    if shutil.which(compiler) is None:
        pytest.skip(f"{compiler} not available")
    exe = str(tmp_path / "walk")
    build = subprocess.run([compiler, *FLAGS, *extra, "-o", exe, os.path.join(ROOT, "tests", "sanitize", src), "-lm"],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ)
    # the sanitizer runtime is linked statically; a preloaded library ahead of it is not an error here
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    report = run.stdout + run.stderr
    assert run.returncode == 0, report
    assert "ERROR: AddressSanitizer" not in report and "runtime error" not in report and "LeakSanitizer" not in report, report
    return report


def test_oracle_under_sanitizers(tmp_path):
    assert "oracle walk ok" in _build_and_run(tmp_path, "gcc", "oracle_driver.c", [])


def test_generators_under_sanitizers(tmp_path):
    assert "generator walk ok" in _build_and_run(tmp_path, "g++", "generators_driver.cpp", ["-std=c++17"])
