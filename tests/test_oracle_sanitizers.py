"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a C++ driver calls every entry
point over seeded random pool life cycles (floating anchors, verification, policies, evictions, span
overflow, both layouts, rotation) and attention matrices; the sanitizers stop at the first bad access,
leak or undefined operation.  Host code only; the GPU library is not involved."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-o", exe, os.path.join(HERE, "oracle_sanitize_driver.cpp"),
           os.path.join(ROOT, "oracle", "cp_oracle.cpp")]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in built.stderr.lower() and "cannot find" in built.stderr.lower():
        pytest.skip("this toolchain has no static AddressSanitizer runtime")
    assert built.returncode == 0, built.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout[-1000:], run.stderr[-3000:])
    assert run.stdout.strip().endswith("done")
