#!/usr/bin/env python3
"""Runs the CPU test suite (`-m "not gpu"`) with the CPU side of the repository built under
AddressSanitizer and UndefinedBehaviorSanitizer: the oracle (oracle/tbe_oracle.c) and the host-only table
assignment solver of the library (csrc/tbe_place.hip, plain C++).  GPU code is not involved.

    python tests/sanitize_cpu_side.py

Builds both into tests/_san/ (not tracked), then starts pytest in a child process with the sanitizer run-times
preloaded (the Python interpreter itself is not instrumented) and TBE_SANITIZED_LIBS pointing there, which makes
tests/conftest.py load these builds.  Any report of either sanitizer ends the run with an error.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "tests", "_san")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def main() -> int:
    os.makedirs(OUT, exist_ok=True)
    subprocess.check_call(["gcc", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"] + SAN +
                          ["-o", os.path.join(OUT, "libtbe_oracle_san.so"), os.path.join(ROOT, "oracle", "tbe_oracle.c"), "-lm"])
    subprocess.check_call(["g++", "-std=c++17", "-x", "c++", "-fPIC", "-shared", "-Wall"] + SAN +
                          ["-o", os.path.join(OUT, "libtbe_place_san.so"),
                           os.path.join(ROOT, "paper_2305_01515_amd", "csrc", "tbe_place.hip")])
    rt = [subprocess.check_output(["gcc", "-print-file-name=" + n], text=True).strip() for n in ("libasan.so", "libubsan.so")]
    env = dict(os.environ, TBE_SANITIZED_LIBS=OUT, LD_PRELOAD=":".join(rt + [os.environ.get("LD_PRELOAD", "")]).strip(":"),
               ASAN_OPTIONS="detect_leaks=0:halt_on_error=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    return subprocess.call([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests"), "-x", "-q", "-m", "not gpu"] + sys.argv[1:],
                           env=env, cwd=ROOT)


if __name__ == "__main__":
    sys.exit(main())
