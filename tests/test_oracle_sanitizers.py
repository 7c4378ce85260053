"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU):
oracle/sanitize_driver.c calls every entry point on small odd-sized inputs with buffers of
exactly the documented sizes; any out-of-bounds access, leak of a per-call allocation, signed
overflow or misaligned access aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan",
           os.path.join(ROOT, "oracle", "tokfilt_oracle.c"),
           os.path.join(ROOT, "oracle", "sanitize_driver.c"), "-lm", "-o", exe]
    subprocess.check_call(cmd)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "runtime error" not in r.stderr and "ERROR: AddressSanitizer" not in r.stderr, r.stderr
    assert "checksum" in r.stdout
