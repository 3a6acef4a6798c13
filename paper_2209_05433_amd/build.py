"""Builds libfp8mm.so (the HIP kernels and their C ABI) and libfp8probes.so (the measurement probes
of bench.py) for gfx950 with hipcc, in-tree.

Every translation unit is compiled to an object of its own, in parallel; the tiled GEMM source is
compiled eight times, once per pair of operand storage orders (-DFP8MM_LAYOUT=0..3) and
accumulation mode (-DFP8MM_ACC=0|1)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libfp8mm.so")
PROBES_LIB = os.path.join(PKG, "libfp8probes.so")     # measurement probes for bench.py, not part of the product library

# (source, extra defines, object name)
UNITS = [("gemm_tiled.hip", ["-DFP8MM_LAYOUT=%d" % k, "-DFP8MM_ACC=%d" % a], "gemm_tiled_l%d_a%d.o" % (k, a))
         for k in range(4) for a in range(2)] + \
        [("gemm_dispatch.hip", [], "gemm_dispatch.o"), ("gemm_splitk.hip", [], "gemm_splitk.o"), ("gemm_mfma_any.hip", [], "gemm_mfma_any.o"),
         ("cast_kernels.hip", [], "cast_kernels.o"),
         ("cast_variants.hip", [], "cast_variants.o"),
         ("api.hip", [], "api.o")]

# -packed-fp32-ops is switched off on purpose: the compiler must not form packed fp32
# instructions from the scalar float code of the kernels.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    """Compile every source every time it is called; returns the path of the library."""
    os.makedirs(OBJ, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    jobs = [[hipcc(), *HIPCC_FLAGS, *inc, *defs, "-c", os.path.join(CSRC, src), "-o", os.path.join(OBJ, obj)]
            for src, defs, obj in UNITS]
    jobs.append([hipcc(), *HIPCC_FLAGS, *inc, "-shared", os.path.join(CSRC, "probes.hip"), "-o", PROBES_LIB])
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB,
          *[os.path.join(OBJ, obj) for _, _, obj in UNITS]], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
