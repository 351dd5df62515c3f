"""The host side of the library under AddressSanitizer + UndefinedBehaviorSanitizer (host code only; no GPU is
used): argument validation of every entry point and the decode planner's integer arithmetic over shapes up to
the limits of the integer types (tests/host/abi_sanitize.cpp).  A sanitizer report or a wrong status fails the run."""
import os
import subprocess

from paper_2406_03482_amd import build


def test_validation_and_planner_are_clean_under_host_sanitizers():
    exe = build.build_host_sanitizer_driver()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert r.stdout.strip().endswith("ok")
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
