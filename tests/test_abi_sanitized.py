"""The host side of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU).

`python -m paper_2311_09550_amd.build --host-sanitize` compiles the library with its host code instrumented (the device
code as usual) and links `tests/abi_selftest.c` against it; the driver exercises the host packer on exact-size heap
blocks, the size and planning functions over the extremes of the contract, and the argument checks of every launching
entry point.  The build recompiles every kernel (about two minutes), so this test runs only when asked to:
W4A8_HOST_SANITIZE=1 python -m pytest tests/test_abi_sanitized.py"""
import os
import subprocess

import pytest


@pytest.mark.skipif(os.environ.get("W4A8_HOST_SANITIZE") != "1",
                    reason="recompiles the whole library with host sanitizers (two minutes): set W4A8_HOST_SANITIZE=1")
def test_abi_host_side_is_clean_under_asan_and_ubsan():
    from paper_2311_09550_amd.build import build_host_sanitized
    exe = build_host_sanitized()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "abi selftest ok" in r.stdout
