"""The engine's host code (slot table, page allocator, update protocol, packing helper) compiled with
AddressSanitizer and UndefinedBehaviorSanitizer and driven, without a GPU, by tests/host/sanitize_driver.c
through the C ABI on bookkeeping-only engines.  Sanitizers cover host code only."""
import os
import subprocess

import pytest

from paper_2509_19128_amd import build as plbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_logic_is_clean_under_asan_and_ubsan(tmp_path):
    try:
        exe = plbuild.build_sanitized_driver(os.path.join(ROOT, "tests", "host", "sanitize_driver.c"), str(tmp_path))
    except plbuild.SanitizerUnavailable as ex:
        pytest.skip(str(ex))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    report = r.stdout + r.stderr
    assert r.returncode == 0, report[-4000:]
    assert "AddressSanitizer" not in report and "runtime error" not in report and "LeakSanitizer" not in report, report[-4000:]
    assert "host logic clean under the sanitizers" in r.stdout
