"""Small driver for profiler runs (rocprofv3 --kernel-trace / --pmc): launches a plain copy of
known size (the calibration kernel for HBM byte counters) and then the kernels of one workload a
few times, with random FP8 bytes / bf16 values already resident in HBM.

    python3 -m paper_2209_05433_amd.profile_run --workload ffn_up_175b --mode f16 --iters 3
    python3 -m paper_2209_05433_amd.profile_run --workload quantize_only --iters 3
    python3 -m paper_2209_05433_amd.profile_run --workload cast_variants --iters 3
"""
from __future__ import annotations

import argparse

import torch

from . import binding as fp8

SHAPES = {  # name: (M, N, K, fmtA, out dtype)
    "ffn_up_175b": (8192, 49152, 12288, 0, torch.bfloat16),
    "dgrad_175b": (8192, 12288, 49152, 1, torch.float32),
    "small_gpt_fwd": (4096, 6144, 2048, 0, torch.bfloat16),
}


def random_codes(shape, top=0x5F):
    mag = torch.randint(0, top + 1, shape, dtype=torch.uint8, device="cuda")
    return mag | (torch.randint(0, 2, shape, dtype=torch.uint8, device="cuda") << 7)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="ffn_up_175b", choices=sorted(SHAPES) + ["quantize_only", "cast_variants"])
    ap.add_argument("--mode", default="f16", choices=["f16", "mfma8"])
    ap.add_argument("--iters", type=int, default=3)
    ap.add_argument("--copy-mib", type=int, default=1024, help="size of the calibration copy")
    ap.add_argument("--mnk", type=int, nargs=3, default=None, help="GEMM shape overriding the workload's")
    ap.add_argument("--trans-a", type=int, default=0, help="1: A stored K x M")
    ap.add_argument("--trans-b", type=int, default=0, help="1: B stored N x K")
    args = ap.parse_args()

    n = args.copy_mib << 20
    src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)                         # reads n bytes, writes n bytes
    torch.cuda.synchronize()
    del src, dst

    if args.workload == "quantize_only":
        m = 1 << 28
        x = torch.randn(m, device="cuda").to(torch.bfloat16)
        q = torch.empty(m, dtype=torch.uint8, device="cuda")
        amax = torch.zeros(1, device="cuda")
        scale = torch.zeros(1, device="cuda")
        for _ in range(args.iters):
            fp8.fp8_amax(x, amax)
            for fmt in (fp8.FP8_E4M3, fp8.FP8_E5M2):
                fp8.fp8_scale_from_amax(amax, fmt, scale)
                fp8.fp8_quantize_dscale(x, fmt, scale, q)
    elif args.workload == "cast_variants":
        rows = cols = 1 << 14
        x = torch.randn(rows * cols, device="cuda").to(torch.bfloat16).view(rows, cols)
        q = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
        qt = torch.empty((cols, rows), dtype=torch.uint8, device="cuda")
        amax = torch.zeros(1, device="cuda")
        scale = torch.ones(1, device="cuda")
        row_amax, row_scale = torch.zeros(rows, device="cuda"), torch.ones(rows, device="cuda")
        for _ in range(args.iters):
            fp8.fp8_quantize_amax(x.view(-1), fp8.FP8_E4M3, scale, q.view(-1), amax)
            fp8.fp8_quantize_sr(x.view(-1), fp8.FP8_E4M3, scale, 1234, q.view(-1))
            fp8.fp8_quantize_transpose(x, fp8.FP8_E4M3, scale, q, qt)
            fp8.fp8_amax_rows(x, row_amax)
            fp8.fp8_quantize_rows(x, fp8.FP8_E4M3, row_scale, q)
    else:
        M, N, K, fmtA, out = SHAPES[args.workload]
        if args.mnk:
            M, N, K = args.mnk
        A = random_codes((K, M) if args.trans_a else (M, K))
        B = random_codes((N, K) if args.trans_b else (K, N))
        C = torch.empty((M, N), dtype=out, device="cuda")
        flags = 0 if args.mode == "f16" else fp8.FP8_GEMM_MFMA8
        for _ in range(args.iters):
            fp8.fp8_gemm_ex(A, fmtA, args.trans_a, B, fp8.FP8_E4M3, args.trans_b, C, 1.0, 1.0, flags)
    torch.cuda.synchronize()


if __name__ == "__main__":
    main()
