"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer.

The oracle's C source is compiled together with tests/sanitize_oracle.c (a
brute-force battery over every schedule on every small configuration) with
-fsanitize=address,undefined and run as a plain executable, so no sanitizer
runtime has to be loaded into the Python process.  A report of either sanitizer
aborts the run; a wrong end state or count makes it exit with status 1."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "sanitize_oracle"
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-Wall", "-Wextra", "-I", os.path.join(ROOT, "oracle"),
           os.path.join(ROOT, "oracle", "bcast_oracle.c"), os.path.join(ROOT, "tests", "sanitize_oracle.c"), "-lm", "-o", str(exe)]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, "exit %d\n%s\n%s" % (run.returncode, run.stdout[-2000:], run.stderr[-4000:])
    assert "0 failures" in run.stdout, run.stdout
