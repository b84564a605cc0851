"""The host side of the library (argument validation, split planning, error text: csrc/hb_api.hip)
built with AddressSanitizer and UndefinedBehaviorSanitizer and driven through its error paths by a
small C program (tests/host_sanitize_driver.c).  Runs without a GPU: no call reaches a launch."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_shim_under_address_and_undefined_behaviour_sanitizers():
    sys.path.insert(0, ROOT)
    from paper_2509_18824_amd import build as B
    exe = B.build_host_sanitizer_check(os.path.join(ROOT, "tests", "host_sanitize_driver.c"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out
    assert "host shim checks passed" in out
    assert "AddressSanitizer" not in out and "runtime error" not in out, out
