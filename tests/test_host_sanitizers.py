"""The library's host-only code (partitioner, bidirectional partitioner, schedule simulation, bubble filling,
hyper-parameter search, error messages) built as plain C++ under AddressSanitizer and UndefinedBehaviorSanitizer
and driven through seeded random problems, error paths and sizes at the guards (tests/host_sanitize_driver.cpp).
No GPU and no GPU code is involved."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which(os.environ.get("CXX", "g++")) is None, reason="no host C++ compiler")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    from paper_2405_01248_amd import build
    exe = build.build_host_sanitized(os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), str(tmp_path / "host_sanitize_driver"))
    # verify_asan_link_order=0: the environment may preload a library of its own ahead of the sanitizer runtime
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    print(r.stdout[-2000:], r.stderr[-4000:])
    assert r.returncode == 0, r.stderr[-4000:]
    assert "host sanitizer driver: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
