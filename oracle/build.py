"""Compile the C oracle into oracle/libscalekv_oracle.so with gcc.

Test infrastructure only: building the checker is not using it.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, n) for n in ("scalekv_oracle.c", "selection_literal.c", "allocation.c")]
LIB = os.path.join(HERE, "libscalekv_oracle.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in SRCS):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-ffp-contract=off", "-o", LIB] + SRCS + ["-lm"]
    subprocess.run(cmd, check=True)
    return LIB


SANITIZE_BIN = os.path.join(HERE, "sanitize_check")


def build_sanitized() -> str:
    """The oracle sources and their driver (sanitize_main.c) as one executable with
    AddressSanitizer and UndefinedBehaviorSanitizer, every report fatal."""
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra",
           "-ffp-contract=off", "-o", SANITIZE_BIN] + SRCS + [os.path.join(HERE, "sanitize_main.c"), "-lm"]
    subprocess.run(cmd, check=True)
    return SANITIZE_BIN


def run_sanitized() -> str:
    """Build and run the sanitizer executable; returns its output, raises if it reports anything."""
    exe = build_sanitized()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    out = res.stdout + res.stderr
    if res.returncode != 0 or "runtime error" in out or "Sanitizer" in out:
        raise RuntimeError("the sanitizer build of the oracle reported a problem:\n" + out)
    return out


if __name__ == "__main__":
    import sys
    if "--sanitize" in sys.argv:
        print(run_sanitized().strip())
    else:
        print(build(force=True))
