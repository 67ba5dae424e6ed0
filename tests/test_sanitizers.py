"""Sanitizer builds, on the CPU only: the oracle under AddressSanitizer + UndefinedBehavior-
Sanitizer with all of its pins, and the host-only logic of the C ABI (planner, argument and
threshold validation that returns before the first GPU call) in a plain C++ program linked
with stand-ins for the kernel launchers.  GPU code is never instrumented."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def gcc_file(name):
    return subprocess.run(["gcc", "-print-file-name=" + name], check=True, capture_output=True,
                          text=True).stdout.strip()


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    asan = gcc_file("libasan.so")
    if not os.path.isabs(asan):
        pytest.skip("no libasan.so next to gcc")
    env = dict(os.environ, GAC_ORACLE_LIB=str(tmp_path / "libgac_oracle_san.so"),
               GAC_ORACLE_CXXFLAGS=" ".join(SAN),
               # the instrumented library is loaded into an uninstrumented python: the runtime
               # has to come first; python's own leaks at exit are not the oracle's
               LD_PRELOAD=":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x),
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "passed" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
    assert os.path.exists(env["GAC_ORACLE_LIB"]), "the instrumented copy was not what ran"


def test_host_logic_of_the_c_abi_under_asan_and_ubsan(tmp_path):
    hip_inc = "/opt/rocm/include"
    hip_lib = "/opt/rocm/lib"
    if shutil.which("g++") is None or not os.path.exists(os.path.join(hip_inc, "hip", "hip_runtime_api.h")):
        pytest.skip("needs g++ and the HIP runtime headers")
    exe = tmp_path / "host_check"
    cmd = ["g++", "-std=c++17", "-Wall"] + SAN + [
        "-D__HIP_PLATFORM_AMD__", "-I", hip_inc, "-I", os.path.join(ROOT, "include"),
        "-I", os.path.join(ROOT, "paper_2603_01501_amd", "csrc"),
        os.path.join(ROOT, "paper_2603_01501_amd", "csrc", "gac_api.cpp"),
        os.path.join(ROOT, "tests", "host_check.cpp"), "-o", str(exe),
        "-L", hip_lib, "-lamdhip64", "-Wl,-rpath," + hip_lib]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stdout + b.stderr
    # (a preloaded library in the environment may come before the sanitizer runtime: allowed)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "host checks ok" in r.stdout, r.stdout[-3000:] + r.stderr[-3000:]
