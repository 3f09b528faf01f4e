"""The host side of the library under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

The packer (tsvd_pack.cpp: format, bit manipulation, threads, validation of untrusted blobs) is built with g++ and both
sanitizers together with a driver that exercises round trips on ragged shapes, every error path and corrupted blobs;
a sanitizer report aborts the driver.  GPU code cannot be run under sanitizers here, so the device entry points'
argument checks are covered by tests/test_abi_host.py instead."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_packer_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitizer_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-pthread", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           os.path.join(ROOT, "tests", "host", "sanitizer_driver.cpp"),
           os.path.join(ROOT, "paper_2308_07641_amd", "csrc", "tsvd_pack.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    # (the environment is passed on unchanged; verify_asan_link_order=0 lets the runtime start when a preloaded
    # library precedes it in the process)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "host sanitizer driver: ok" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
