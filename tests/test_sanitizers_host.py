"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU oracle and of the library's host-only code
(schedulers, partition controller, split selection, input validation), each run as a small driver program: any
report makes the program exit non-zero.  GPU code is not involved (the two host-only translation units of the
library build with a plain C++ compiler)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
# (verify_asan_link_order=0: the environment may preload a library of its own ahead of the sanitizer runtime)
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")


def _run(cmd, exe):
    r = subprocess.run(cmd, capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 0, f"build failed:\n{r.stderr[-4000:]}"
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, cwd=ROOT)
    assert r.returncode == 0, f"{exe} failed (sanitizer report or check):\n{r.stdout[-2000:]}\n{r.stderr[-6000:]}"
    assert "ok" in r.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-std=c11", "-fopenmp", "-Wall", *SAN, "-o", exe, os.path.join(ROOT, "tests", "san", "oracle_driver.c"), "-lm"], exe)


def test_host_side_library_code_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_san")
    csrc = os.path.join(ROOT, "paper_2507_06608_amd", "csrc")
    _run(["g++", "-std=c++17", "-Wall", *SAN, "-o", exe, "-x", "c++", os.path.join(csrc, "nexus_host.hip"), "-x", "c++",
          os.path.join(csrc, "nexus_sched.hip"), "-x", "c++", os.path.join(ROOT, "tests", "san", "host_driver.cpp")], exe)
