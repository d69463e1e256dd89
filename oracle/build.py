"""Compile the C oracle into oracle/liboracle.so with plain gcc.

Test infrastructure only.  No fast-math, no FMA contraction: every fp32
operation of the quantiser must be a single IEEE-754 operation.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "gqsa_oracle.c")
# (GQSA_ORACLE_LIBRARY: the sanitizer leg of the tests loads the build below instead)
LIB = os.environ.get("GQSA_ORACLE_LIBRARY") or os.path.join(HERE, "liboracle.so")
SANITIZED_LIB = os.path.join(HERE, "liboracle_asan.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
           "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
           SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized() -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (gcc's)."""
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-Wall", "-Wextra", SRC, "-o", SANITIZED_LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return SANITIZED_LIB


def sanitizer_runtime() -> str:
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()


if __name__ == "__main__":
    print(build())
