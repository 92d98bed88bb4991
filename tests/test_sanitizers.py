"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, nothing touches a
GPU): the oracle is rebuilt with both sanitizers and its pins run against that build in a
child process; the library's host-side launch arithmetic runs under them too.  A report from
either sanitizer (out-of-bounds access, signed overflow, misaligned load, shift out of range,
...) fails the test."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
REPORT_MARKS = ("ERROR: AddressSanitizer", "runtime error:", "SUMMARY: UndefinedBehaviorSanitizer")


def gcc_runtime(name):
    path = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    libasan = gcc_runtime("libasan.so")
    if not libasan:
        pytest.skip("gcc's libasan.so not found")
    lib = str(tmp_path / "liboracle_san.so")
    build = subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fPIC", "-shared",
                            "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                            "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", lib,
                            os.path.join(ROOT, "oracle", "scar_oracle.c"), "-lm"],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ)
    env.update({"SCAR_ORACLE_LIB": lib, "LD_PRELOAD": libasan,
                # the Python interpreter itself is not leak-clean; leaks are not what is looked for
                "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1",
                "OMP_NUM_THREADS": "4"})
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True)
    text = run.stdout + run.stderr
    assert run.returncode == 0, text[-4000:]
    for mark in REPORT_MARKS:
        assert mark not in text, text[-4000:]
    assert " passed" in run.stdout


def test_host_launch_arithmetic_under_asan_and_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "host_logic_san")
    # sanitizers on the host pass only: each -fsanitize option directly after -Xarch_host
    build = subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-w",
                            "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                            "-Xarch_host", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                            os.path.join(ROOT, "tests", "host", "host_logic.cpp"), "-o", exe],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0"
    run = subprocess.run([exe], env=env, capture_output=True, text=True)
    text = run.stdout + run.stderr
    assert run.returncode == 0, text[-3000:]
    assert "host logic ok" in run.stdout
    for mark in REPORT_MARKS:
        assert mark not in text, text[-3000:]
