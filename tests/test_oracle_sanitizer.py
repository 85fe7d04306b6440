"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, gcc).

The oracle's loops index tapes by series, position, layer and unit; a stray index would still give
plausible numbers.  This builds oracle/esrnn_oracle.c with -fsanitize=address,undefined together with a
driver (tests/oracle_sanitizer_main.c) that calls every entry point on ragged, seasonal, non-seasonal,
double-seasonal and degenerate shapes, and requires a clean exit.  No GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_is_clean_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fopenmp", "-Wall", "-Wextra",
           os.path.join(ROOT, "oracle", "esrnn_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitizer_main.c"),
           "-o", exe, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ)
    # (link-order check off: a library preloaded by the environment may come before the sanitizer runtime)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "2"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + "\n" + r.stderr
    assert "FAILED" not in r.stdout and r.stdout.count(" ok ") == 9, r.stdout
