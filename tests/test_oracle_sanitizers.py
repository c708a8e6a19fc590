"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host only, no GPU): every
oracle function on small ragged and degenerate shapes with exact-size heap operands."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
@pytest.mark.parametrize("real", ["double", "float"])
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path, real):
    exe = str(tmp_path / f"sanitize_check_{real}")
    # the sanitizer runtimes are linked statically, so that the program does not depend on the order of
    # the libraries an environment may preload
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",
           "-fno-omit-frame-pointer", f"-DORACLE_REAL={real}", "-I", os.path.join(ROOT, "oracle"),
           os.path.join(ROOT, "oracle", "sanitize_check.c"), "-o", exe, "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle sanitize check: ok" in run.stdout and "ERROR" not in run.stderr
