"""Host code of the library under the address and undefined-behaviour sanitizers (no GPU needed): builds
csrc/_build_asan/host_checks (python -m paper_1706_07191_amd.build --host-asan) and runs it.  The program walks
argument validation, working-set sizing, block resolution, the launch planners over thousands of shapes and the
failure paths of the calls that need a device; any out-of-bounds access, signed overflow, or memory still held
at exit makes it exit non-zero."""
import os
import shutil
import subprocess

import pytest

from paper_1706_07191_amd import build as builder


def test_host_code_is_clean_under_asan_and_ubsan():
    if not (os.path.exists("/opt/rocm/bin/hipcc") or shutil.which("hipcc")):
        pytest.skip("hipcc not available")
    exe = builder.build_host_asan()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "0 failed" in r.stdout and "ERROR" not in r.stderr
