"""Address and undefined-behaviour sanitizers over the CPU-side code: the C oracle (every entry point, through
tests/sanitize/oracle_driver.c) and the library's host code (the C ABI's validation, planning and host
algorithms, through tests/sanitize/abi_driver.cpp; device code is compiled as usual, only the host pass is
instrumented).  Both are standalone executables so that the sanitizer runtime comes first in their own process."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "tests", "sanitize", "_build")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(exe):
    p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=ENV, timeout=300)
    assert p.returncode == 0, p.stdout[-4000:]
    return p.stdout


def test_oracle_under_address_and_ub_sanitizers():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_san")
    subprocess.check_call(["gcc", "-std=c99", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-Wall", "-o", exe, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                           os.path.join(ROOT, "oracle", "ic_oracle.c"), "-lm"])
    assert "oracle sanitizer run ok" in _run(exe)


def test_library_host_code_under_address_and_ub_sanitizers():
    sys.path.insert(0, ROOT)
    from paper_2603_12201_amd import build as lib_build
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "abi_san")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all", "-g"]
    objs = lib_build.compile_objects(extra=san, tag=".san")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-std=c++17", "-I" + os.path.join(ROOT, "include")] + san +
                          ["-x", "c++", os.path.join(ROOT, "tests", "sanitize", "abi_driver.cpp"), "-x", "none"] + objs +
                          ["-o", exe])
    assert "abi sanitizer run ok" in _run(exe)
