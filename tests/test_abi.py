"""CPU-only checks of the boundary: the built library loads, exports what include/fp8mm.h
declares, and rejects bad arguments before touching the GPU.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2209_05433_amd as fp8

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "fp8mm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fp8_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = fp8.lib()
    names = declared_symbols()
    assert set(names) == set(fp8.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_binding_has_the_same_names():
    for n in declared_symbols():
        assert callable(getattr(fp8, n)), n


def test_header_is_plain_c_and_a_c_program_links(tmp_path):
    """include/fp8mm.h must compile as C and as C++ without HIP or torch headers, and a C program
    must link against the library and get an error status for a bad call (nothing is launched)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "use.c"
    src.write_text(
        '#include <stdio.h>\n#include <string.h>\n#include "fp8mm.h"\n'
        "int main(void) {\n"
        "    float cell = 0.0f;\n"
        "    int st = fp8_amax(&cell, 4, 99, &cell, 0);          /* bad dtype: rejected on the host */\n"
        '    printf("%d %s|%s\\n", st, fp8_version(), fp8_last_error());\n'
        "    return st == FP8_ERR_INVALID_ARG && strstr(fp8_last_error(), \"in_dtype\") ? 0 : 1;\n"
        "}\n")
    for cc, std in (("gcc", "-std=c99"), ("g++", "-std=c++11")):
        if shutil.which(cc) is None:
            continue
        unit = tmp_path / ("hdr_" + cc + (".c" if cc == "gcc" else ".cpp"))
        unit.write_text('#include "fp8mm.h"\nint unused_symbol_of_this_unit;\n')
        subprocess.run([cc, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, "-c", str(unit), "-o", str(unit) + ".o"],
                       check=True, capture_output=True, text=True)
    libdir = os.path.dirname(fp8.LIB_PATH)
    exe = tmp_path / "use"
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-lfp8mm", "-Wl,-rpath," + libdir],
                   check=True, capture_output=True, text=True)
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "gfx950" in res.stdout


def test_gemm_plan_names_the_kernel_for_the_workload_shapes():
    """fp8_gemm_plan is host logic over shapes, storage orders and pointer alignment (no pointer is
    dereferenced, so made-up aligned addresses do): the five workloads and the layer GEMMs around them
    must land on the tiled matrix-core kernel, and only shapes it cannot take on the any-shape one."""
    L = fp8.lib()
    A, B, C = 1 << 20, 1 << 24, 1 << 28                         # 16-byte aligned stand-ins
    T256, T128, ANY, EW = fp8.FP8_PLAN_TILED_256x256, fp8.FP8_PLAN_TILED_256x128, fp8.FP8_PLAN_MFMA_ANY, fp8.FP8_PLAN_ELEMENTWISE_STORES
    plan = lambda ta, tb, M, N, K, a=A, b=B, c=C, sb=None: L.fp8_gemm_plan(a, ta, b, tb, c, M, N, K, sb)
    assert plan(0, 0, 8192, 49152, 12288) == T256                # config 4
    assert plan(1, 0, 8192, 12288, 49152) == T256                # config 5 with A stored K x M
    assert plan(0, 0, 4096, 6144, 2048) == T128 | fp8.FP8_PLAN_PERSISTENT   # config 3: 384 wide tiles would leave half a round empty;
                                                                            # 768 narrow ones = 3 per compute unit, walked as one K loop
    assert not plan(0, 0, 4096, 6144 + 16, 2048) & fp8.FP8_PLAN_PERSISTENT   # an edge tile: one workgroup per tile
    assert plan(0, 0, 4096, 6144, 2048 + 64) == T128             # K not in whole stage pairs
    assert plan(0, 0, 4096, 6144, 8192) == fp8.FP8_PLAN_TILED_MIXED   # long K: 256 wide tiles, then 256 narrow ones, one launch
    assert plan(0, 0, 256, 256, 256) in (T256, T128)             # config 1
    for ta in (0, 1):
        for tb in (0, 1):
            assert plan(ta, tb, 12288, 49152, 8192) == T256      # weight gradient of the FFN-up layer, any storage order
    assert plan(0, 1, 8192, 50257, 12288) == T256 | EW           # vocabulary-sized N with weights stored [out, in]
    assert plan(0, 0, 8192, 50257, 12288) == ANY                 # ... stored [in, out]: rows of B start anywhere: the any-shape matrix-core kernel
    assert plan(1, 0, 50257, 12288, 8192) == ANY                 # rows of an M-contiguous A start anywhere
    assert plan(0, 0, 512, 512, 448) in (T256, T128)             # K = 7 stages of 64: the last stage pair is half zeros
    assert plan(0, 0, 8192, 12288, 12352) == T256                # K = 64 x odd
    assert plan(0, 1, 8192, 12288, 12304) == T256                # K a multiple of 16 only
    assert plan(0, 0, 512, 512, 440) == ANY                      # K not a multiple of 16: rows of A start anywhere
    assert plan(0, 0, 512, 512, 512, a=A + 4) == ANY             # operand not 16-byte aligned
    assert plan(0, 0, 4096, 4096, 512, c=C + 2) == T256 | EW     # output not 16-byte aligned
    assert plan(0, 0, 4096, 4096, 512, sb=C + 4) == T256 | EW    # per-column factors not 16-byte aligned
    assert plan(0, 0, 0, 5, 5) == fp8.FP8_PLAN_NO_GEMM and plan(0, 0, 5, 5, 0) == fp8.FP8_PLAN_NO_GEMM
    assert plan(2, 0, 5, 5, 5) == -fp8.FP8_ERR_INVALID_ARG and plan(0, 0, -1, 5, 5) == -fp8.FP8_ERR_INVALID_ARG


def test_knobs_round_trip_and_reject_bad_values():
    assert fp8.fp8_get_knob(fp8.FP8_KNOB_TILE_N) == 0
    assert fp8.fp8_set_knob(fp8.FP8_KNOB_TILE_N, 128) == 0
    assert fp8.fp8_get_knob(fp8.FP8_KNOB_TILE_N) == 128
    L = fp8.lib()
    A, B, C = 1 << 20, 1 << 24, 1 << 28
    assert L.fp8_gemm_plan(A, 0, B, 0, C, 8192, 49152, 12288, None) == fp8.FP8_PLAN_TILED_256x128
    assert fp8.fp8_set_knob(fp8.FP8_KNOB_TILE_N, 0) == 128
    assert L.fp8_gemm_plan(A, 0, B, 0, C, 8192, 49152, 12288, None) == fp8.FP8_PLAN_TILED_256x256
    assert fp8.fp8_set_knob(fp8.FP8_KNOB_GEMM_KERNEL, 1) == 0
    assert L.fp8_gemm_plan(A, 0, B, 0, C, 8192, 49152, 12288, None) == fp8.FP8_PLAN_FMA_KERNEL
    assert L.fp8_gemm_plan(A, 0, B, 0, C, 512, 500, 77, None) == fp8.FP8_PLAN_FMA_KERNEL
    assert fp8.fp8_set_knob(fp8.FP8_KNOB_GEMM_KERNEL, 2) == 1
    assert L.fp8_gemm_plan(A, 0, B, 0, C, 8192, 49152, 12288, None) == fp8.FP8_PLAN_MFMA_ANY
    fp8.fp8_set_knob(fp8.FP8_KNOB_GEMM_KERNEL, 0)
    assert fp8.fp8_set_knob(fp8.FP8_KNOB_MIXED, 1) == 0
    assert L.fp8_gemm_plan(A, 0, B, 0, C, 4096, 6144, 2048, None) == fp8.FP8_PLAN_TILED_256x128 | fp8.FP8_PLAN_PERSISTENT
    assert fp8.fp8_set_knob(fp8.FP8_KNOB_MIXED, 2) == 1
    assert L.fp8_gemm_plan(A, 0, B, 0, C, 8192, 49152, 12288, None) == fp8.FP8_PLAN_TILED_MIXED
    fp8.fp8_set_knob(fp8.FP8_KNOB_MIXED, 0)
    assert L.fp8_gemm_plan(A, 0, B, 0, C, (1 << 31) * 128, 128 * 3, 77, None) == fp8.FP8_PLAN_FMA_KERNEL   # more 128 x 128 tiles than a grid holds
    for knob, bad in ((fp8.FP8_KNOB_TILE_N, 64), (fp8.FP8_KNOB_CAST_PATH, 2), (fp8.FP8_KNOB_SPLIT_K, 65), (fp8.FP8_KNOB_GEMM_KERNEL, 3), (99, 0)):
        with pytest.raises(fp8.Fp8Error):
            fp8.fp8_set_knob(knob, bad)


def test_splitk_workspace_size_is_slices_times_the_fp32_output():
    size = fp8.fp8_gemm_splitk_workspace_size
    assert size(1024, 1024, 65536, 1, 0, 0) == 16 * 1024 * 1024 * 4        # 16 tiles -> 16 slices of 32 stage pairs
    assert size(1024, 1024, 65536, 1, 0, 8) == 8 * 1024 * 1024 * 4
    assert size(1024, 1024, 65536, 1, 0, 1) == 0                           # one slice: the plain kernel, no workspace
    assert size(8192, 49152, 12288, 0, 0, 0) == 0                          # enough tiles to fill the chip
    assert size(256, 256, 256, 0, 0, 0) == 0                               # too short a K to cut
    assert size(256, 256, 300, 0, 0, 4) == 0                               # not a problem of the tiled kernel
    assert size(256, 256, 384, 0, 0, 64) == 3 * 256 * 256 * 4              # never more slices than stage pairs
    assert size(0, 5, 5, 0, 0, 0) == 0 and size(5, 5, 5, 0, 0, 65) == 0
    L = fp8.lib()
    buf = (ctypes.c_float * 64)()
    p = ctypes.addressof(buf)
    INV = fp8.FP8_ERR_INVALID_ARG
    assert L.fp8_gemm_splitk(p, 0, 0, p, 0, 0, p, 4, 4, 4, 0, 1.0, 1.0, None, None, 0, 65, None, 0, None) == INV
    assert L.fp8_gemm_splitk(p, 0, 0, p, 0, 0, p, 4, 4, 4, 0, 1.0, 1.0, None, None, 0, 2, p + 2, 64, None) == INV
    assert L.fp8_gemm_splitk(p, 0, 0, p, 0, 0, p, 1024, 1024, 65536, 0, 1.0, 1.0, None, None, 0, 8, p, 64, None) == INV
    assert "workspace of 33554432 bytes" in fp8.fp8_last_error()


def test_version_and_error_strings():
    assert "gfx950" in fp8.fp8_version()
    L = fp8.lib()
    assert L.fp8_amax(None, 4, 0, None, None) == fp8.FP8_ERR_INVALID_ARG
    assert "amax_out" in fp8.fp8_last_error()


def test_invalid_arguments_are_rejected_without_a_launch():
    L = fp8.lib()
    buf = (ctypes.c_float * 64)()
    p = ctypes.addressof(buf)
    INV = fp8.FP8_ERR_INVALID_ARG
    assert L.fp8_amax(p, 4, 7, p, None) == INV                       # bad dtype
    assert L.fp8_amax(None, 4, 0, p, None) == INV                    # null x, n > 0
    assert L.fp8_amax(p + 2, 4, 0, p, None) == INV                   # misaligned fp32
    assert L.fp8_scale_from_amax(None, 0, p, None) == INV
    assert L.fp8_scale_from_amax(p, 5, p, None) == INV
    assert L.fp8_quantize(p, 4, 0, 9, 1.0, p, None) == INV           # bad format
    assert L.fp8_quantize(p, 4, 3, 0, 1.0, p, None) == INV           # bad dtype
    assert L.fp8_quantize(None, 4, 0, 0, 1.0, p, None) == INV
    assert L.fp8_quantize(p, 0, 0, 0, 1.0, None, None) == fp8.FP8_OK  # n == 0 launches nothing
    assert L.fp8_quantize_dscale(p, 4, 0, 0, None, p, None) == INV
    assert L.fp8_quantize_ex(p, 4, 0, 0, 1.0, None, 2, p, None) == INV          # unknown flag
    assert L.fp8_quantize_ex(p, 4, 0, 0, 1.0, p + 2, 0, p, None) == INV       # misaligned device scale
    assert L.fp8_dequantize(p, 4, 3, 1.0, None, 0, p, None) == INV
    assert L.fp8_dequantize(p, 4, 0, 1.0, None, 0, None, None) == INV
    assert L.fp8_dequantize(None, 0, 0, 1.0, None, 1, None, None) == fp8.FP8_OK
    assert L.fp8_gemm(p, 0, 1.0, p, 0, 1.0, p, -1, 4, 4, 0, None) == INV
    assert L.fp8_gemm(p, 2, 1.0, p, 0, 1.0, p, 4, 4, 4, 0, None) == INV
    assert L.fp8_gemm(p, 0, 1.0, p, 0, 1.0, p, 4, 4, 4, 5, None) == INV
    assert L.fp8_gemm(None, 0, 1.0, p, 0, 1.0, p, 4, 4, 4, 0, None) == INV
    assert L.fp8_gemm(p, 0, 1.0, p, 0, 1.0, None, 4, 4, 4, 0, None) == INV
    assert L.fp8_gemm(p, 0, 1.0, p, 0, 1.0, p, 0, 4, 4, 0, None) == fp8.FP8_OK   # empty output
    assert L.fp8_gemm_dscale(p, 0, None, p, 0, p, p, 4, 4, 4, 0, None) == INV
    assert "scale pointer" in fp8.fp8_last_error()
    assert L.fp8_gemm_ex(p, 0, 2, p, 0, 0, p, 4, 4, 4, 0, 1.0, 1.0, None, None, 0, None) == INV     # transA not 0/1
    assert L.fp8_gemm_ex(p, 0, 0, p, 0, 0, p, 4, 4, 4, 0, 1.0, 1.0, p, None, 0, None) == INV        # one scale on device only
    assert L.fp8_gemm_ex(p, 0, 0, p, 0, 0, p, 4, 4, 4, 0, 1.0, 1.0, None, None, 8, None) == INV     # unknown flag
    fused = lambda **kw: L.fp8_gemm_fused(*[kw.get(k, d) for k, d in (
        ("A", p), ("fmtA", 0), ("transA", 0), ("B", p), ("fmtB", 0), ("transB", 0), ("D", p), ("out_kind", 2),
        ("M", 4), ("N", 4), ("K", 4), ("sA", p), ("nsA", 1), ("sB", p), ("nsB", 4), ("sD", None), ("amax", None),
        ("flags", 0), ("stream", None))])
    assert fused(out_kind=4) == INV
    assert fused(nsA=3) == INV and "nsA" in fp8.fp8_last_error()
    assert fused(nsB=2) == INV
    assert fused(sA=None) == INV
    assert fused(out_kind=1, sD=p) == INV                                        # output scale with a bf16 output
    assert fused(amax=p + 2) == INV
    assert fused(D=None) == INV
    assert fused(M=0) == fp8.FP8_OK


@pytest.mark.parametrize("fmt", [fp8.FP8_E4M3, fp8.FP8_E5M2])
def test_host_scale_rule_matches_the_oracle(fmt):
    rng = np.random.default_rng(17)
    vals = np.concatenate([2.0 ** rng.uniform(-140, 127, 4000),
                           [0.0, 1.0, 448.0, 57344.0, np.inf, np.nan, 1e-45, 3.4e38]]).astype(np.float32)
    for a in vals:
        got = np.float32(fp8.fp8_scale_from_amax_host(float(a), fmt))
        assert got == oracle.scale_from_amax(a, fmt), float(a)
    assert fp8.fp8_scale_from_amax_host(1.0, 3) == 1.0 and "fmt" in fp8.fp8_last_error()


def test_binding_refuses_host_tensors():
    import torch
    x = torch.zeros(8)
    with pytest.raises(ValueError):
        fp8.fp8_amax(x, torch.zeros(1))


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more must end with a message, before anything is run."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
