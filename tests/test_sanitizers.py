"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the library's plan
and schedule tables (plan.cpp) over the cluster shapes of the host tests, and the oracle's C
arithmetic on ragged lengths with exactly sized buffers."""
import os
import subprocess

import pytest

from test_plan_host import SHAPES

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1",
       "-static-libasan", "-static-libubsan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _build(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and ("-static-libasan" in r.stderr or "libasan" in r.stderr or "libubsan" in r.stderr):
        pytest.skip("this toolchain has no static sanitizer runtimes: " + r.stderr.strip().splitlines()[-1])
    assert r.returncode == 0, r.stderr


def test_plan_tables_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "plan_san")
    csrc = os.path.join(ROOT, "paper_2310_06003_amd", "csrc")
    _build(["g++", "-std=c++17", "-Wall", *SAN, "-I", os.path.join(ROOT, "include"), "-I", csrc,
            os.path.join(csrc, "plan.cpp"), os.path.join(ROOT, "tests", "sanitize", "plan_main.cpp"), "-o", exe,
            "-lpthread"])
    shapes = [f"{P}:{G}" for P, G in SHAPES] + ["256:16", "3:1", "12:12"]
    r = subprocess.run([exe, *shapes], capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "failures 0" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_oracle_arithmetic_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _build(["gcc", "-std=c11", "-Wall", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", *SAN,
            os.path.join(ROOT, "oracle", "update.c"), os.path.join(ROOT, "tests", "sanitize", "oracle_main.c"), "-o", exe,
            "-lm"])
    r = subprocess.run([exe], capture_output=True, text=True, env=dict(ENV, OMP_NUM_THREADS="4"), timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "oracle sanitizer run ok" in r.stdout and "runtime error" not in r.stderr
