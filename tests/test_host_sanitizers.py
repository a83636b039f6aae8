"""The host-side C++ of the library (argument validation, reorder index, bitmask -> block list,
launch schedule) built with AddressSanitizer + UndefinedBehaviorSanitizer and run on the CPU: the
sanitizers abort the program on any out-of-bounds access, leak or undefined operation."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_host_api_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_api_sanitized")
    cmd = [HIPCC, "-x", "hip", "--offload-arch=gfx950", "-std=c++17", "-O1", "-g",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2506_16054_amd", "csrc"),
           os.path.join(ROOT, "paper_2506_16054_amd", "csrc", "host_api.cpp"), os.path.join(ROOT, "tests", "host_api_sanitized.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert build.returncode == 0, build.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120, env=env)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "host api under sanitizers: ok" in run.stdout
