"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host-side code: the CPU oracle (plain C) and the
library's host scheduler with its scripted test backend (C++).  Each is compiled together with a driver under
tests/sanitize/ that walks its entry points and edge cases, and must run through with no report.  Host code
only: nothing here touches a GPU, and the sanitizer runtimes are linked statically into the drivers."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan",
       "-fno-omit-frame-pointer", "-g", "-O1", "-Wall", "-Wextra"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:allocator_may_return_null=1",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")


def _build_and_run(cmd, exe):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert p.returncode == 0, p.stdout
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=ENV, timeout=600)
    assert r.returncode == 0, f"exit status {r.returncode}\n{r.stdout}\n{r.stderr[-4000:]}"
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr and "LeakSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    out = _build_and_run(["gcc", "-std=c11", "-fopenmp"] + SAN + ["-o", exe, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                                                                 os.path.join(ROOT, "oracle", "adadecode_oracle.c"), "-lm"], exe)
    assert "ran through" in out


def test_host_scheduler_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sched_san")
    csrc = os.path.join(ROOT, "paper_2506_03700_amd", "csrc")
    out = _build_and_run(["g++", "-std=c++17"] + SAN + ["-o", exe, os.path.join(ROOT, "tests", "sanitize", "sched_driver.cpp"),
                                                        os.path.join(csrc, "ad_sched.cpp"), os.path.join(csrc, "ad_sched_testhook.cpp")], exe)
    assert "runs through" in out
