"""The host side of the library (pool bookkeeping, plan builder, exports, models) under
AddressSanitizer and UndefinedBehaviorSanitizer: a small C++ driver is compiled together with the
library sources, sanitizers on the host pass only, and run on the CPU.  It makes no device call."""
import glob
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_abi_host_paths_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc here")
    exe = str(tmp_path / "tl_host_sanitize")
    srcs = sorted(glob.glob(os.path.join(ROOT, "paper_2508_17219_amd", "csrc", "*.hip")))
    cmd = [hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2508_17219_amd", "csrc"),
           os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp")] + srcs + ["-o", exe]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-3000:]
    assert "all statuses as expected" in run.stdout and "runtime error" not in run.stdout, run.stdout[-3000:]
