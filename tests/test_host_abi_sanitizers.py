"""The entry points' host code (argument validation, workspace arithmetic, dispatch: csrc/api.hip and
csrc/decode_noalloc.hip) under AddressSanitizer and UndefinedBehaviorSanitizer, no GPU: a second build of
the library with those two files' host side instrumented runs tests/test_host_abi.py in a child process.
Every call that file makes fails validation before anything is launched, so no kernel runs."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not available")
def test_host_validation_is_clean_under_asan_and_ubsan(tmp_path):
    from paper_2412_12094_amd import build

    runtime = build.sanitizer_runtime()
    if not runtime:
        pytest.skip("no shared sanitizer runtime next to the compiler")
    lib = build.build_host_sanitized(str(tmp_path / "libsepattn_hostsan.so"))
    pre = os.environ.get("LD_PRELOAD", "")
    env = dict(os.environ, SEPATTN_LIB=lib, LD_PRELOAD=runtime + (":" + pre if pre else ""),
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_host_abi.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)
    out = run.stdout + run.stderr
    assert run.returncode == 0, out[-4000:]
    assert "passed" in run.stdout and "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    # the child did load the instrumented build
    probe = subprocess.run([sys.executable, "-c",
                            "import paper_2412_12094_amd as sp, ctypes; lib = sp.load(); print(sp.LIB_PATH); "
                            "print(open('/proc/self/maps').read().count('libsepattn_hostsan'))"],
                           capture_output=True, text=True, env=env, cwd=ROOT, timeout=300)
    assert probe.returncode == 0 and lib in probe.stdout and int(probe.stdout.split()[-1]) > 0, probe.stdout + probe.stderr
