"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer.

tests/sanitize_driver.cpp is compiled together with every source of the library -- the
sanitizers on the host pass only (the device code is built as usual) -- and run here: host
coarsening of 60 random graphs with every accessor, plans, orders, schedules, the tuning
record and the argument checks, with no device call, so no GPU is needed.  About a minute
and a half, nearly all of it compilation."""
import os
import shutil
import subprocess

import pytest

from paper_2008_12336_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(900)
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_driver")
    san = []
    for flag in ("-fsanitize=address", "-fsanitize=undefined", "-fno-omit-frame-pointer"):
        san += ["-Xarch_host", flag]
    cmd = [B.hipcc(), "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fopenmp", "-munsafe-fp-atomics",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *san,
           "-I" + os.path.join(ROOT, "include"), "-I" + B.CSRC, "-x", "hip",
           *[os.path.join(B.CSRC, s) for s in B.SOURCES], os.path.join(ROOT, "tests", "sanitize_driver.cpp"),
           "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "asan driver ok" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
