"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only: gcc).

tests/oracle_sanitizer_driver.c calls every exported routine of oracle/fp8_oracle.c on empty, tiny
and ragged inputs (specials included) and prints one checksum per routine.  It is built twice
with the oracle's source, once plainly and once with -fsanitize=address,undefined (reports are
fatal); the sanitized run must end without a report and print the checksums of the plain one."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = [os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c"), os.path.join(ROOT, "oracle", "fp8_oracle.c")]


def build(tmp_path, name, flags):
    exe = str(tmp_path / name)
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-fopenmp", *flags, "-o", exe, *SRC, "-lm"],
                       capture_output=True, text=True)
    if r.returncode != 0 and "sanitize" in " ".join(flags) and ("cannot find" in r.stderr or "unrecognized" in r.stderr):
        pytest.skip("this gcc has no sanitizer runtime: " + r.stderr.strip().splitlines()[-1])
    assert r.returncode == 0, r.stderr
    return exe


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    plain = build(tmp_path, "plain", ["-O2"])
    san = build(tmp_path, "san", ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"])
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    want = subprocess.run([plain], capture_output=True, text=True, timeout=300, env=env)
    assert want.returncode == 0 and len(want.stdout.split()) == 10, want.stdout + want.stderr
    got = subprocess.run([san], capture_output=True, text=True, timeout=600, env=env)
    assert got.returncode == 0, got.stdout + got.stderr
    assert "runtime error" not in got.stderr and "AddressSanitizer" not in got.stderr and "LeakSanitizer" not in got.stderr, got.stderr
    assert got.stdout == want.stdout
