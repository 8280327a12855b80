"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code that has no GPU in it: the
library's block-list builder (rf_plan.cpp) and the C oracle (rf_oracle.c), driven by
tests/sanitize_driver.cpp on the CogVideoX-, Open-Sora-Plan- and HunyuanVideo-shaped layouts and
on degenerate ones, at blocks 64 / 128 / 256."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# the sanitizer runtimes are linked statically, so a library preloaded into every process cannot come before them
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1", "-static-libasan",
       "-static-libubsan"]


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs gcc and g++")
def test_plan_builder_and_oracle_run_clean_under_asan_and_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_2505_21036_amd", "csrc")
    oracle_o = str(tmp_path / "rf_oracle.o")
    exe = str(tmp_path / "sanitize_driver")
    # the oracle without OpenMP: its pragmas are then ignored and every loop runs on this thread
    subprocess.check_call(["gcc", "-std=c11", "-c", os.path.join(ROOT, "oracle", "rf_oracle.c"), "-o", oracle_o] + SAN)
    subprocess.check_call(["g++", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", csrc,
                           os.path.join(ROOT, "tests", "sanitize_driver.cpp"), os.path.join(csrc, "rf_plan.cpp"), oracle_o,
                           "-o", exe, "-lm"] + SAN)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitize ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stdout + r.stderr
