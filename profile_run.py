"""Small driver for profiler runs (rocprofv3 --kernel-trace / --pmc): launches a plain copy of
known size (the calibration kernel for HBM byte counters) and then the kernels of one workload a
few times, on the data bench.py times (--data synth: the workload's seeded synthetic tensors, cast
to FP8 by the library itself) or on uniformly random FP8 codes (--data random).

    python3 profile_run.py --workload ffn_up_175b --mode f16 --iters 3
    python3 profile_run.py --workload quantize_only --iters 3
    python3 profile_run.py --workload cast_variants --iters 3
    python3 profile_run.py --workload splitk --iters 6
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2209_05433_amd as fp8
from workloads import synth

SHAPES = {  # name: (M, N, K, fmtA, out dtype, generator)
    "ffn_up_175b": (8192, 49152, 12288, 0, torch.bfloat16, synth.config4),
    "dgrad_175b": (8192, 12288, 49152, 1, torch.float32, synth.config5),
    "small_gpt_fwd": (4096, 6144, 2048, 0, torch.bfloat16, synth.config3),
}


def synth_codes(gen, M, N, K, fmtA, trans_a, trans_b):
    """The workload's tensors, cast on the device with per-tensor amax scaling as in bench.py."""
    A_bits, B_bits = gen(M, N, K)
    ws = torch.zeros(fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
    amax, scale = torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
    out = []
    for bits, fmt in ((A_bits, fmtA), (B_bits, fp8.FP8_E4M3)):
        x = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
        q = torch.empty(bits.shape, dtype=torch.uint8, device="cuda")
        fp8.fp8_amax_scale(x, fmt, amax, scale, ws)
        fp8.fp8_quantize_dscale(x, fmt, scale, q)
        torch.cuda.synchronize()
        out.append(q)
    A, B = out
    return (A.t().contiguous() if trans_a else A), (B.t().contiguous() if trans_b else B)


def random_codes(shape, top=0x5F):
    mag = torch.randint(0, top + 1, shape, dtype=torch.uint8, device="cuda")
    return mag | (torch.randint(0, 2, shape, dtype=torch.uint8, device="cuda") << 7)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="ffn_up_175b", choices=sorted(SHAPES) + ["quantize_only", "cast_variants", "splitk"])
    ap.add_argument("--mode", default="f16", choices=["f16", "mfma8"])
    ap.add_argument("--iters", type=int, default=3)
    ap.add_argument("--ramp", type=int, default=12, help="untimed GEMM launches first (clock ramp after idle), as in bench.py")
    ap.add_argument("--copy-mib", type=int, default=1024, help="size of the calibration copy")
    ap.add_argument("--mnk", type=int, nargs=3, default=None, help="GEMM shape overriding the workload's")
    ap.add_argument("--trans-a", type=int, default=0, help="1: A stored K x M")
    ap.add_argument("--trans-b", type=int, default=0, help="1: B stored N x K")
    ap.add_argument("--data", default="synth", choices=["synth", "random"], help="GEMM operands: the workload's synthetic tensors or uniform codes")
    args = ap.parse_args()

    n = args.copy_mib << 20
    src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)                         # reads n bytes, writes n bytes
    torch.cuda.synchronize()
    del src, dst

    if args.workload == "quantize_only":
        m = 1 << 28
        h = synth.config2(m)
        x = torch.from_numpy(h.view(np.int16)).view(torch.bfloat16).cuda()
        q = torch.empty(m, dtype=torch.uint8, device="cuda")
        amax = torch.zeros(1, device="cuda")
        scale = torch.zeros(1, device="cuda")
        ws = torch.zeros(fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
        for _ in range(args.iters):
            for fmt in (fp8.FP8_E4M3, fp8.FP8_E5M2):
                fp8.fp8_amax_scale(x, fmt, amax, scale, ws)
                fp8.fp8_quantize_dscale(x, fmt, scale, q)
    elif args.workload == "splitk":
        # the weight-gradient regime of bench.py: 1024 x 1024 x 65536, A stored K x M; one workgroup per tile, then K slices
        M = N = 1024
        K = 65536
        A, B = random_codes((K, M), 0x4F), random_codes((K, N), 0x6F)
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        ws = torch.empty(max(fp8.fp8_gemm_splitk_workspace_size(M, N, K, 1, 0, 0), 16), dtype=torch.uint8, device="cuda")
        flags = 0 if args.mode == "f16" else fp8.FP8_GEMM_MFMA8
        for _ in range(args.iters):
            fp8.fp8_gemm_ex(A, fp8.FP8_E5M2, 1, B, fp8.FP8_E4M3, 0, C, 1.0, 1.0, flags)
        for _ in range(args.iters):
            fp8.fp8_gemm_splitk(A, fp8.FP8_E5M2, 1, B, fp8.FP8_E4M3, 0, C, 1.0, 1.0, ws, flags, 0)
    elif args.workload == "cast_variants":
        rows = cols = 1 << 14
        x = torch.randn(rows * cols, device="cuda").to(torch.bfloat16).view(rows, cols)
        q = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
        qt = torch.empty((cols, rows), dtype=torch.uint8, device="cuda")
        amax = torch.zeros(1, device="cuda")
        scale = torch.ones(1, device="cuda")
        row_amax, row_scale = torch.zeros(rows, device="cuda"), torch.ones(rows, device="cuda")
        yb = torch.empty(rows * cols, dtype=torch.bfloat16, device="cuda")
        yf = torch.empty(rows * cols, dtype=torch.float32, device="cuda")
        for _ in range(args.iters):
            fp8.fp8_quantize_amax(x.view(-1), fp8.FP8_E4M3, scale, q.view(-1), amax)
            fp8.fp8_quantize_sr(x.view(-1), fp8.FP8_E4M3, scale, 1234, q.view(-1))
            fp8.fp8_quantize_transpose(x, fp8.FP8_E4M3, scale, q, qt)
            fp8.fp8_amax_rows(x, row_amax)
            fp8.fp8_quantize_rows(x, fp8.FP8_E4M3, row_scale, q)
            fp8.fp8_dequantize(q.view(-1), fp8.FP8_E4M3, scale, yb)
            fp8.fp8_dequantize(q.view(-1), fp8.FP8_E4M3, scale, yf)
    else:
        M, N, K, fmtA, out, gen = SHAPES[args.workload]
        if args.mnk:
            M, N, K = args.mnk
        if args.data == "synth":
            A, B = synth_codes(gen, M, N, K, fmtA, args.trans_a, args.trans_b)
        else:
            A = random_codes((K, M) if args.trans_a else (M, K))
            B = random_codes((N, K) if args.trans_b else (K, N))
        C = torch.empty((M, N), dtype=out, device="cuda")
        flags = 0 if args.mode == "f16" else fp8.FP8_GEMM_MFMA8
        for _ in range(args.ramp + args.iters):
            fp8.fp8_gemm_ex(A, fmtA, args.trans_a, B, fp8.FP8_E4M3, args.trans_b, C, 1.0, 1.0, flags)
    torch.cuda.synchronize()


if __name__ == "__main__":
    main()
