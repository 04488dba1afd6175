"""The C oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (host only) and driven over
ragged shapes, every depth, scales, value maps and the rounding routines by a small C program; any
out-of-bounds access, signed overflow or misaligned access aborts it.  No GPU needed."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no gcc")
def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", exe,
           os.path.join(HERE, "oracle_sanitizer_driver.c"), os.path.join(ROOT, "oracle", "msgemm_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)  # the sanitizer runtime wants to be first; nothing else is needed in this process
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "oracle sanitizer driver: ok" in r.stdout
