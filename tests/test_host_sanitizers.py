"""The host side of libkvp (validation, layout, the state machine of Alg. 1, launch planning)
built without the device code and with -fsanitize=address,undefined, driven through its C ABI by
tests/host_asan/driver.cpp.  Any out-of-bounds access, use after free, overflow or misaligned
access in those paths aborts the driver."""
import os
import shutil
import subprocess

import pytest

from paper_2604_16734_amd.build import build_host_sanitized


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_state_machine_under_asan_and_ubsan(tmp_path):
    exe = build_host_sanitized(str(tmp_path))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
