"""The host-only code of the library (Step I of the reordering, the schedule, the Matrix Market
reader) and the oracle, compiled with AddressSanitizer and UndefinedBehaviorSanitizer and run on
seeded inputs (tests/host_sanitized_driver.cpp).  CPU only; device code is not part of this build."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = shutil.which("amdclang++") or "/opt/rocm/llvm/bin/clang++"


@pytest.mark.skipif(not os.path.exists(CLANG), reason="no clang++ with sanitizer runtimes")
def test_host_stages_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "host_sanitized"
    csrc = os.path.join(ROOT, "paper_2501_09251_amd", "csrc")
    sources = [os.path.join(ROOT, "tests", "host_sanitized_driver.cpp"), os.path.join(csrc, "reorder.cpp"),
               os.path.join(csrc, "schedule.cpp"), os.path.join(csrc, "mtx.cpp"), os.path.join(ROOT, "oracle", "oracle.cpp")]
    cmd = [CLANG, "-x", "c++", "-std=c++17", "-O1", "-g", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
           "-I", os.path.join(ROOT, "include"), "-I", csrc, "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-Wno-unknown-pragmas"] + sources + ["-o", str(exe)]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    run = subprocess.run([str(exe), str(tmp_path)], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "host stages clean" in run.stdout
