"""Host code of the library under AddressSanitizer + UndefinedBehaviorSanitizer (GPU sanitizers are not available here).

The instrumented build takes a few minutes, so this test runs when the executable is already there and newer than the
sources (`python -m paper_2210_17323_amd.build --host-sanitize` makes it), or when GPTQ_HOST_SANITIZE=1 asks for the build.
"""
import os
import subprocess

import pytest

from paper_2210_17323_amd import build as B


def test_c_abi_validation_paths_are_clean_under_host_sanitizers():
    if os.environ.get("GPTQ_HOST_SANITIZE") == "1" and not B.host_sanitized_is_current():
        B.build_host_sanitized(verbose=False)
    if not B.host_sanitized_is_current():
        pytest.skip("no current host-sanitized build (python -m paper_2210_17323_amd.build --host-sanitize, or GPTQ_HOST_SANITIZE=1)")
    env = dict(os.environ, UBSAN_OPTIONS="print_stacktrace=1", ASAN_OPTIONS="detect_leaks=0")
    p = subprocess.run([B.SAN_BIN], capture_output=True, text=True, env=env, timeout=120)
    assert p.returncode == 0, p.stdout + p.stderr
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr, p.stderr
    assert "host ABI checks passed" in p.stdout
