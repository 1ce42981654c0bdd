"""CPU sanitizer tier: the host-only pass planner and the CPU oracle compiled with
-fsanitize=address,undefined (g++, no HIP involved) and driven by tests/sanitize_host.cpp over a
sweep of small cases.  Any report (heap overflow, use after free, signed overflow, bad shift,
misaligned access ...) aborts the program and fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVER = os.path.join(ROOT, "tests", "sanitize_host.cpp")
FLAGS = ["-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
         "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan"]


def build_and_run(tmp_path, name, define, sources, extra):
    if shutil.which("g++") is None:
        pytest.skip("g++ not available")
    exe = str(tmp_path / name)
    cmd = ["g++"] + FLAGS + ["-D" + define] + extra + [DRIVER] + sources + ["-o", exe]
    subprocess.check_call(cmd)
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)               # the sanitizer runtime must come first
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:exitcode=23"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "2"
    r = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600)
    assert r.returncode == 0, "sanitized %s failed (rc %d)\n%s\n%s" % (name, r.returncode, r.stdout, r.stderr[-4000:])
    assert "clean" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_planner_under_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2602_13140_amd", "csrc")
    build_and_run(tmp_path, "san_planner", "SANITIZE_PLANNER", [os.path.join(csrc, "qsv_plan.cpp")],
                  ["-I", csrc, "-I", os.path.join(ROOT, "include")])


def test_oracle_under_sanitizers(tmp_path):
    build_and_run(tmp_path, "san_oracle", "SANITIZE_ORACLE", [os.path.join(ROOT, "oracle", "qsv_oracle.cpp")],
                  ["-fopenmp"])
