"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a second build of oracle/rdk_oracle.c, linked
with a driver that takes every oracle function through a small, exactly sized problem.  A read or write past an array,
a signed overflow or a misaligned access in the oracle aborts the driver with a report."""
import os
import subprocess

ORACLE_DIR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    build = subprocess.run(
        ["gcc", "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-ffp-contract=off", "-fsanitize=address,undefined",
         "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan",
         os.path.join(ORACLE_DIR, "rdk_oracle.c"), os.path.join(ORACLE_DIR, "sanitize_driver.c"), "-o", exe, "-lm"],
        capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120,
                         env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1"))
    assert run.returncode == 0, run.stdout + run.stderr
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
    assert "every oracle function ran clean" in run.stdout
