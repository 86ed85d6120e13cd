"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a small
C driver (tests/oracle_sanitized_driver.c) calls every entry point on ragged
layouts with exactly sized heap buffers.  Skipped where gcc has no static
sanitizer runtimes."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_runs_clean_under_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_san")
    cmd = [gcc, "-std=c99", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           os.path.join(ROOT, "oracle", "ef_oracle.c"), os.path.join(HERE, "oracle_sanitized_driver.c"),
           "-lm", "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and ("libasan" in built.stderr or "libubsan" in built.stderr):
        pytest.skip("sanitizer runtimes not installed: " + built.stderr.strip().splitlines()[-1])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle sanitized run ok" in run.stdout
