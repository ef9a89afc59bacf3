"""CPU-side sanitizer runs (no GPU): the oracle under AddressSanitizer + UndefinedBehaviorSanitizer
through a driver that calls every one of its functions, and the host code of the library (argument
validation, workspace layouts, error reporting) under the same sanitizers through a driver that makes
only calls the host answers before any launch.  HCTR_SANITIZE=1 additionally builds the oracle that
the Python tests load with UndefinedBehaviorSanitizer (oracle.build)."""
import os
import subprocess

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan():
    out = oracle.sanitize_check()
    assert "sanitize driver: clean" in out


def test_host_side_of_the_library_is_clean_under_asan_and_ubsan():
    from paper_2210_08803_amd import build
    exe = build.build_host_sanitized(os.path.join(ROOT, "tests", "abi_sanitize_driver.cpp"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1")   # the HIP runtime's own start-up allocations are not ours
    done = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert done.returncode == 0, done.stdout + done.stderr
    assert "abi sanitize driver: clean" in done.stdout
