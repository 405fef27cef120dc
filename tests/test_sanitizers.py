"""The host-side C / C++ of this build under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU involved): the CPU
oracle and the dispatching code are each compiled into a small driver (tests/sanitize/) with
-fsanitize=address,undefined -fno-sanitize-recover=all; the drivers exercise every entry point, the full / empty /
argument-error paths included, and must exit cleanly without a sanitizer report or a leak."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
FLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]


def build_and_run(tmp_path, compiler, std, src, extra):
    exe = str(tmp_path / (os.path.splitext(src)[0] + "_san"))
    cmd = [compiler, std, *FLAGS, *extra, os.path.join(HERE, "sanitize", src), "-o", exe, "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in built.stderr.lower() and "cannot find" in built.stderr.lower():
        pytest.skip("the sanitizer runtime libraries are not installed with this compiler")
    assert built.returncode == 0, built.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    report = run.stdout[-1500:] + run.stderr[-3000:]
    assert run.returncode == 0, report
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr and "LeakSanitizer" not in run.stderr, report
    assert "checksum" in run.stdout
    return run.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    build_and_run(tmp_path, "gcc", "-std=c11", "oracle_driver.c", ["-fopenmp"])


def test_dispatch_code_under_asan_ubsan(tmp_path):
    build_and_run(tmp_path, "g++", "-std=c++17", "dispatch_driver.cpp", ["-I", os.path.join(ROOT, "include")])
