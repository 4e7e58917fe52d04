"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer -- CPU only.

oracle/sanitize_main.c calls every entry point of the oracle on small ragged inputs; here it is built
with -fsanitize=address,undefined and run.  A heap overrun, a leak, a misaligned or overflowing
operation anywhere in the oracle ends the program with a report and a non-zero status."""
import os
import shutil
import subprocess

import pytest

ORACLE_DIR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    build = subprocess.run(
        ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-fno-omit-frame-pointer", "-static-libasan", "-std=c11", "-Wall", "-Wextra", "-o", exe,
         os.path.join(ORACLE_DIR, "sanitize_main.c"), "-lm"],
        capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
    assert "0 unexpected return codes" in run.stdout
