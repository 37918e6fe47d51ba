"""The library's HOST code -- argument checks, workspace planning, kernel choice, launch shapes
of every entry point -- built with AddressSanitizer and UndefinedBehaviorSanitizer and driven
over seeded problem sizes.  HIP calls are stubs that succeed (tests/hip_launch_stub.h, force-
included), so nothing here needs a GPU; the kernels themselves are not compiled (--cuda-host-only)."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_library_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitized")
    csrc = os.path.join(ROOT, "paper_2504_19232_amd", "csrc")
    srcs = sorted(glob.glob(os.path.join(csrc, "*.hip")))
    assert len(srcs) >= 5
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]
    cmd = [HIPCC, "--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17", *san,
           "-Wno-unused-command-line-argument", "-Wno-int-to-pointer-cast",
           "-include", os.path.join(ROOT, "tests", "hip_launch_stub.h"), "-I", os.path.join(ROOT, "include"), "-I", csrc,
           "-x", "hip", *srcs, os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "runtime error" not in run.stderr and "ERROR: AddressSanitizer" not in run.stderr, run.stderr[-4000:]
    assert run.stdout.startswith("checksum ")
