"""The library's host code (argument validation, schedule helpers, accounting) under AddressSanitizer
and UndefinedBehaviorSanitizer: the sources are rebuilt with the sanitizers on the HOST side only and
linked with a driver that walks the error paths (nothing is launched, so no GPU is needed)."""
import os
import subprocess

import pytest

from conftest import ROOT
from paper_2412_20105_amd import build


@pytest.mark.timeout(900)
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = build.build_host_sanitized(os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), str(tmp_path / "st3_host_san"))
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"      # the HIP runtime keeps its own allocations
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=600)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert r.returncode == 0, tail
    assert "0 failures" in r.stdout, tail
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, tail
