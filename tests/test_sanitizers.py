"""Sanitizer leg of the CPU side: the host code of the library (packer, image builders, C
boundary; the device side stubbed out) and the C oracle, each rebuilt with AddressSanitizer and
UndefinedBehaviorSanitizer and driven by the same CPU tests as the ordinary builds, in a child
process that has the sanitizer's runtime preloaded.  GPU code is neither compiled nor sanitized here.
"""
from __future__ import annotations

import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_under(runtime, extra_env, test_files):
    env = dict(os.environ)
    env.update(extra_env)
    # the sanitizer's runtime must come first among the preloaded libraries; whatever is
    # preloaded already stays
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter itself is not instrumented: its own allocations at exit are not ours to judge
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *test_files]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    report = r.stdout[-4000:] + r.stderr[-4000:]
    assert r.returncode == 0, report
    assert "ERROR: AddressSanitizer" not in report and "runtime error:" not in report, report
    assert " passed" in r.stdout, report


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers():
    from paper_2412_17560_amd import build as lib_build
    lib = lib_build.build_sanitized()
    runtime = lib_build.sanitizer_runtime()
    if not os.path.exists(runtime):
        pytest.skip(f"no AddressSanitizer runtime at {runtime}")
    _run_under(runtime, {"GQSA_LIBRARY": lib}, ["tests/test_pack_bitexact.py", "tests/test_abi.py"])


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    from oracle import build as oracle_build
    lib = oracle_build.build_sanitized()
    runtime = oracle_build.sanitizer_runtime()
    if not os.path.exists(runtime):
        pytest.skip(f"no AddressSanitizer runtime at {runtime}")
    _run_under(runtime, {"GQSA_ORACLE_LIBRARY": lib}, ["tests/test_oracle_pins.py", "tests/test_oracle_layout.py"])
