"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a C++ driver that reaches the
arithmetic's edges (INT32 extremes through every shift, wrapping sums, padded taps, NaN and huge
reals, empty tensors) is built together with oracle/hago_ref.cpp with both sanitizers on and has to
run to the end without a report."""
import os
import subprocess

from conftest import ROOT


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           os.path.join(ROOT, "tests", "oracle_sanitize_driver.cpp"), os.path.join(ROOT, "oracle", "hago_ref.cpp"),
           "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle sanitizer driver: ok" in r.stdout
