"""The C oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (host code only) and
driven over small seeded inputs: the checker itself must be free of heap errors, leaks and
undefined integer behaviour."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    srcs = [os.path.join(ROOT, "oracle", "adaptra_oracle.c"), os.path.join(ROOT, "oracle", "zb_oracle.c"),
            os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c")]
    build = subprocess.run(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                            "-fno-omit-frame-pointer", "-o", exe] + srcs + ["-lpthread"],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "runtime error" not in run.stderr and "ERROR: AddressSanitizer" not in run.stderr, run.stderr
    assert run.stdout.startswith("checksum ")
