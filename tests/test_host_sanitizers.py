"""The host side of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU, no kernel launch).

csrc/api.hip - context, argument checks, workspace layout, the weight re-packing and operand-table builders - is
compiled with the sanitizers on the host pass only and linked with tests/host_sanitize/driver.hip, which stubs the
kernel launchers and walks the same calls as test_host_api.py plus ap_set_weights for every compiled channel pair.
Any report from either sanitizer aborts the driver (non-zero exit)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BUILD = os.path.join(ROOT, "_build")
EXE = os.path.join(BUILD, "host_api_sanitized")

COMMAND = [
    "hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
    "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
    "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
    "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2502_04077_amd", "csrc"),
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    os.path.join(ROOT, "paper_2502_04077_amd", "csrc", "api.hip"),
    os.path.join(ROOT, "tests", "host_sanitize", "driver.hip"), "-o", EXE,
]


def test_host_boundary_is_clean_under_asan_and_ubsan():
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not available")
    os.makedirs(BUILD, exist_ok=True)
    res = subprocess.run(COMMAND, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([EXE], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "all checks passed" in run.stdout
    assert "AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr
