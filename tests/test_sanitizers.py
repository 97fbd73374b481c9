"""Host sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer, leak detection on) of the CPU oracle and of the
host-side serving policies: each source is compiled together with a small driver under tests/sanitize/ that runs every
entry point on seeded inputs and checks the results for consistency.  GPU code has no sanitizer build on this pool; its
memory safety is covered by the canary test (tests/test_gpu_canary.py) and the bounds checks at the C ABI."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")


def build_and_run(cmd, exe):
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, "sanitizer build failed:\n" + r.stderr[-3000:]
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=600)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "ERROR: AddressSanitizer" not in out and "runtime error" not in out and "LeakSanitizer" not in out, out[-4000:]
    return out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no gcc")
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    out = build_and_run(["gcc", "-std=c11", *SAN, "-fopenmp", os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-o", exe, "-lm"], exe)
    assert "oracle sanitizer driver: ok" in out


@pytest.mark.skipif(shutil.which("g++") is None, reason="no g++")
def test_serving_policies_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "serving_san")
    out = build_and_run(["g++", "-std=c++17", *SAN, os.path.join(ROOT, "paper_2602_22732_amd", "csrc", "serving.cpp"),
                         os.path.join(ROOT, "tests", "sanitize", "serving_driver.cpp"), "-o", exe, "-lpthread"], exe)
    assert "serving sanitizer driver: ok" in out
