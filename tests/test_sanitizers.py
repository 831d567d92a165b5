"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU-side code: the oracle (oracle/qamw_oracle.c) and the
host half of libqamw (csrc/qamw_host.cpp: block rule, sign mask, channel scales, CPU Lloyd trainer, pruned-search
table, polar levels).  Each is compiled together with a small driver (tests/sanitize/) that calls every exported
function on small inputs with exactly sized heap buffers; the run must end with status 0 and no sanitizer report.
GPU code is not covered: sanitizers for it are not available on the GPU machines."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-4000:]
    assert "ERROR: AddressSanitizer" not in out and "runtime error:" not in out and "LeakSanitizer" not in out, out[-4000:]
    return out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    subprocess.check_call(["gcc", *SAN, "-ffp-contract=off", "-std=c99", os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                           os.path.join(ROOT, "oracle", "qamw_oracle.c"), "-o", exe, "-lm"])
    assert "oracle driver ok" in _run(exe)


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_host_library_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_driver")
    subprocess.check_call(["g++", *SAN, "-std=c++17", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"),
                           os.path.join(ROOT, "paper_2605_26339_amd", "csrc", "qamw_host.cpp"), "-o", exe, "-lpthread"])
    assert "host driver ok" in _run(exe)
