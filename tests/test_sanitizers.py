"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU code: the oracle (oracle/skim_oracle.c) and
the host part of the library (csrc/skim_alloc.cpp), each driven by a small program under tests/sanitize/.
Host code only: the kernels are checked by running every parity test at several sizes on the GPU."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
       "-fno-omit-frame-pointer", "-g", "-O1"]


def build_and_run(tmp_path, compiler, src, extra):
    exe = str(tmp_path / "san_driver")
    cmd = [compiler] + SAN + extra + ["-o", exe, os.path.join(HERE, "sanitize", src), "-lm"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-4000:]


def test_oracle_under_asan_ubsan(tmp_path):
    build_and_run(tmp_path, "gcc", "oracle_main.c", ["-std=c11", "-fopenmp", "-ffp-contract=off"])


def test_host_allocator_under_asan_ubsan(tmp_path):
    build_and_run(tmp_path, "g++", "alloc_main.cpp", ["-std=c++17", "-I", os.path.join(ROOT, "include")])
