"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU code of this repository: the fp64
oracle (oracle/razor_oracle.c) and the host-only part of the HIP library (csrc/razor_plan.cpp:
argument checks, the selection table of Algorithm 1, buffer sizes, head selection).  Each is
compiled here with -fsanitize=address,undefined together with a driver from tests/sanitize/ that
walks it over exactly-sized buffers, and run as a process of its own; any report ends the run
with a non-zero status.  (GPU code cannot be sanitized on this machine pool.)"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# the sanitizer runtimes are linked statically, so the programs do not depend on being first in
# the list of loaded libraries
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1",
       "-static-libasan", "-static-libubsan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")


def run_sanitized(cmd, exe, expect):
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr[-3000:]
    ran = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert ran.returncode == 0 and expect in ran.stdout, (ran.stdout[-2000:], ran.stderr[-3000:])


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run_sanitized(["gcc", "-std=c11", "-fopenmp", "-Wall", "-Wextra", *SAN, "-o", exe,
                   os.path.join(ROOT, "tests", "sanitize", "oracle_san.c"),
                   os.path.join(ROOT, "oracle", "razor_oracle.c"), "-lm"], exe, "oracle sanitize ok")


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir("/opt/rocm/include"),
                    reason="g++ or the HIP headers not found")
def test_host_planner_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "plan_san")
    csrc = os.path.join(ROOT, "paper_2407_15891_amd", "csrc")
    run_sanitized(["g++", "-std=c++17", "-Wall", *SAN, "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
                   "-I", csrc, "-isystem", "/opt/rocm/include", "-o", exe,
                   os.path.join(ROOT, "tests", "sanitize", "plan_san.cpp"), os.path.join(csrc, "razor_plan.cpp"),
                   "-L/opt/rocm/lib", "-Wl,-rpath,/opt/rocm/lib", "-lamdhip64"], exe, "plan sanitize ok")
