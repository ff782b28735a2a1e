"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host only, no GPU).

`oracle/selftest.c` calls every exported function of the oracle on ragged shapes with heap buffers of exactly the
documented sizes; an out-of-bounds index, a signed overflow or a misaligned access in the oracle aborts it."""
import os
import subprocess

import pytest

import oracle


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    try:
        exe = oracle.build_selftest(str(tmp_path))
    except (subprocess.CalledProcessError, FileNotFoundError) as e:
        pytest.skip(f"gcc cannot build with -fsanitize=address,undefined here: {e}")
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle selftest ok" in r.stdout
