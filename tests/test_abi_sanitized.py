"""The host side of the C ABI (csrc/zo_abi.cpp: validation, workspace planning, call sequencing) built
for the CPU with AddressSanitizer and UndefinedBehaviorSanitizer and driven through its error paths and
through valid planning calls at the benchmark sizes (tests/abi_sanitize/).  The kernel launchers are
stubs that check every scratch pointer against the workspace; nothing here needs a GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "abi_sanitize")
CSRC = os.path.join(ROOT, "paper_2605_28760_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_abi_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "abi_host_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan", "-D__HIP_PLATFORM_AMD__",
           "-I/opt/rocm/include", "-I" + CSRC, os.path.join(CSRC, "zo_abi.cpp"), os.path.join(SAN, "launch_stubs.cpp"),
           os.path.join(SAN, "abi_host_check.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "0 failed" in run.stdout, run.stdout
