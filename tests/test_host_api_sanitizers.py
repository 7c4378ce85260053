"""The host side of the C ABI (argument checking, workspace sizing, the schedule, error paths)
compiled with AddressSanitizer and UndefinedBehaviorSanitizer on the HOST pass only, and driven
without a GPU by tests/host_api_sanitize_driver.cpp."""
import os
import shutil
import subprocess

import pytest

from paper_2512_07090_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = hip_build.HIPCC


@pytest.mark.skipif(not os.path.exists(HIPCC) or shutil.which("g++") is None, reason="needs hipcc and g++")
def test_host_api_is_clean_under_asan_and_ubsan(tmp_path):
    if not os.path.exists(hip_build.LIB):
        hip_build.build()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
    api_o, drv_o, exe = (str(tmp_path / n) for n in ("api_san.o", "drv.o", "host_api_sanitized"))
    subprocess.check_call([HIPCC, *hip_build.FLAGS, "-O1", "-g", *san, "-I" + os.path.join(ROOT, "include"),
                           "-c", os.path.join(hip_build.CSRC, "tokfilt_api.hip"), "-o", api_o],
                          stderr=subprocess.DEVNULL)
    subprocess.check_call(["g++", "-O1", "-g", "-fsanitize=address,undefined", "-I" + os.path.join(ROOT, "include"),
                           "-c", os.path.join(ROOT, "tests", "host_api_sanitize_driver.cpp"), "-o", drv_o])
    # the kernels' launchers come from the in-tree library; the sanitized entry points of api_o win
    pkg = os.path.dirname(hip_build.LIB)
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", *san, drv_o, api_o, "-L" + pkg,
                           "-l:" + os.path.basename(hip_build.LIB), "-Wl,-rpath," + pkg, "-o", exe],
                          stderr=subprocess.DEVNULL)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0"   # the HIP runtime keeps process-lifetime allocations
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "runtime error" not in r.stderr and "ERROR: AddressSanitizer" not in r.stderr, r.stderr
    assert "0 failures" in r.stdout
