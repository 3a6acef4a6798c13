"""The host side of the C ABI (argument checks, dispatch and split-K planning, knobs, size queries)
under AddressSanitizer and UndefinedBehaviorSanitizer.

Every translation unit of the library is compiled for the host only (no device code, seconds) with
the sanitizers, linked against tests/hip_host_stub.c in place of the HIP runtime (a kernel launch
ends the process there), and driven by tests/api_sanitizer_driver.c: rejected arguments of every
entry point, empty problems, plans and workspace sizes over a seeded sweep of shapes up to 2^36.
The run must print "ok" and no sanitizer report."""
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2209_05433_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def clang(cxx=False):
    path = os.path.join(os.path.dirname(os.path.realpath(B.hipcc())), "..", "lib", "llvm", "bin", "clang++" if cxx else "clang")
    for cand in (path, "/opt/rocm/lib/llvm/bin/" + ("clang++" if cxx else "clang")):
        if os.path.exists(cand):
            return cand
    pytest.skip("no clang beside hipcc")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout + r.stderr
    return r


def test_host_side_of_the_abi_is_clean_under_asan_and_ubsan(tmp_path):
    tmp = str(tmp_path)
    host_san = [flag for s in SAN for flag in ("-Xarch_host", s)]
    jobs = [[B.hipcc(), "--cuda-host-only", "-O1", "-g", "-std=c++17", "-fPIC", *host_san, "-Wno-unused-command-line-argument",
             "-I", os.path.join(ROOT, "include"), "-I", B.CSRC, *defs, "-c", os.path.join(B.CSRC, src), "-o", os.path.join(tmp, obj)]
            for src, defs, obj in B.UNITS]
    with ThreadPoolExecutor(max_workers=4) as ex:
        for r in ex.map(lambda c: subprocess.run(c, capture_output=True, text=True), jobs):
            if r.returncode != 0 and ("libclang_rt" in r.stderr or "unsupported option" in r.stderr):
                pytest.skip("this toolchain has no host sanitizers: " + r.stderr.strip().splitlines()[-1])
            assert r.returncode == 0, r.stderr
    objs = [os.path.join(tmp, obj) for _, _, obj in B.UNITS]
    # the host objects refer to their (absent) device images by per-unit symbol names
    undefined = run(["nm", "-u", *objs]).stdout
    with open(os.path.join(tmp, "fatbin_stub.c"), "w") as f:
        for name in sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", undefined))):
            f.write("const char %s[16] = {0};\n" % name)
    run([clang(), "-c", "-fPIC", os.path.join(tmp, "fatbin_stub.c"), "-o", os.path.join(tmp, "fatbin_stub.o")])
    run([clang(), "-c", "-fPIC", "-O1", "-g", *SAN, os.path.join(ROOT, "tests", "hip_host_stub.c"), "-o", os.path.join(tmp, "hip_host_stub.o")])
    lib = os.path.join(tmp, "libfp8mm_hostsan.so")
    r = subprocess.run([clang(cxx=True), "-shared", "-fPIC", *SAN, "-o", lib, *objs, os.path.join(tmp, "fatbin_stub.o"),
                        os.path.join(tmp, "hip_host_stub.o")], capture_output=True, text=True)
    if r.returncode != 0 and "libclang_rt" in r.stderr:
        pytest.skip("no sanitizer runtime for this clang: " + r.stderr.strip().splitlines()[-1])
    assert r.returncode == 0, r.stderr
    exe = os.path.join(tmp, "api_driver")
    run([clang(), "-std=c99", "-g", "-Wall", "-Wextra", *SAN, "-I", os.path.join(ROOT, "include"),
         os.path.join(ROOT, "tests", "api_sanitizer_driver.c"), "-o", exe, "-L", tmp, "-lfp8mm_hostsan", "-Wl,-rpath," + tmp])
    env = {k: v for k, v in os.environ.items() if not k.startswith("FP8MM_")}
    env.update(ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    got = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert got.returncode == 0 and got.stdout.strip() == "ok", got.stdout + got.stderr
    for mark in ("runtime error", "AddressSanitizer", "LeakSanitizer", "host-only build:"):
        assert mark not in got.stderr, got.stderr
