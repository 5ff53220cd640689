"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

The oracle is the yardstick of every parity test, so a silent out-of-bounds read in it would
be a wrong yardstick.  A C driver (tests/sanitize/oracle_driver.c) runs it through every storage
type, trigger policy, threshold mode and record mode; the sanitizers abort on the first error."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    src = os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")
    build = subprocess.run(
        ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-static-libasan", "-fno-omit-frame-pointer", "-o", exe, src, "-lm", "-lpthread"],
        capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert run.stdout.startswith("checksum ")
