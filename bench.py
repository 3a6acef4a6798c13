#!/usr/bin/env python3
"""Benchmark of the scaled-FP8 matrix multiply path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: amax(A), amax(B), the two scales, cast of A and of B to FP8, the FP8 GEMM
with fp32 accumulation and the unscale epilogue.  The workload is the GPT-175B-like FFN-up
layer (8192 tokens x 12288 -> 49152, bf16 in, E4M3 operands, bf16 out).  One JSON line is
printed; beside the headline it carries the roofline of the dominant kernel, the oracle
timed on the host cores (a baseline, not a target), and the same figures for the
quantize-only workload (2^28 bf16 elements) and the FP8-instruction GEMM variant.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0      # dense fp16/bf16 MFMA, MI355X
PEAK_FP8_TFLOPS = 5000.0       # dense FP8 MFMA
PEAK_HBM_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)     # the chip's clocks settle over the first ~10 GEMM launches
    ap.add_argument("--workload", default="ffn_up_175b", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the quantize-only and FP8-instruction legs")
    return ap.parse_args()


# name -> (config number, M, N, K, fmtA, out dtype name)
WORKLOADS = {
    "ffn_up_175b": (4, 8192, 49152, 12288, 0, "bf16"),
    "dgrad_175b": (5, 8192, 12288, 49152, 1, "f32"),
    "small_gpt_fwd": (3, 4096, 6144, 2048, 0, "bf16"),
}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus %d is not supported, use --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2209_05433_amd as fp8
    from workloads import synth

    fp8.lib()                      # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    cfg, M, N, K, fmtA, out_name = WORKLOADS[args.workload]
    fmtB = fp8.FP8_E4M3
    out_dtype = torch.bfloat16 if out_name == "bf16" else torch.float32
    gen = {3: synth.config3, 4: synth.config4, 5: synth.config5}[cfg]
    t0 = time.time()
    A_bits, B_bits = gen(M, N, K)
    to_dev = lambda h: torch.from_numpy(h.view(np.int16)).view(torch.bfloat16).cuda()
    dA, dB = to_dev(A_bits), to_dev(B_bits)
    t_gen = time.time() - t0

    amax = torch.zeros(2, device="cuda")
    scale = torch.zeros(2, device="cuda")
    qA = torch.empty((M, K), dtype=torch.uint8, device="cuda")
    qB = torch.empty((K, N), dtype=torch.uint8, device="cuda")
    C = torch.empty((M, N), dtype=out_dtype, device="cuda")

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(gemm=fp8.fp8_gemm_dscale, record=None):
        if record is not None:
            record[0].record(stream)
        for t, q, i, f in ((dA, qA, 0, fmtA), (dB, qB, 1, fmtB)):
            fp8.fp8_amax(t, amax[i:i + 1])
            fp8.fp8_scale_from_amax(amax[i:i + 1], f, scale[i:i + 1])
            fp8.fp8_quantize_dscale(t, f, scale[i:i + 1], q)
        if record is not None:
            record[1].record(stream)
        gemm(qA, fmtA, scale[0:1], qB, fmtB, scale[1:2], C)
        if record is not None:
            record[2].record(stream)

    def timed(gemm, steps, warmup):
        for _ in range(warmup):
            step(gemm)
        recs = [(ev(), ev(), ev()) for _ in range(steps)]
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for r in recs:
            step(gemm, r)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_start
        cast_ms = sum(r[0].elapsed_time(r[1]) for r in recs) / steps
        gemm_ms = sum(r[1].elapsed_time(r[2]) for r in recs) / steps
        return wall / steps * 1e3, cast_ms, gemm_ms

    flops = 2.0 * M * N * K
    # The chip's clocks settle over the first dozen GEMM launches after idling (the first ones take
    # 5-20 % longer): one untimed whole step, then untimed GEMM launches, precede the W warm-up steps.
    CLOCK_RAMP_LAUNCHES = 12
    step()
    for _ in range(CLOCK_RAMP_LAUNCHES):
        fp8.fp8_gemm_dscale(qA, fmtA, scale[0:1], qB, fmtB, scale[1:2], C)
    ms_step, cast_ms, gemm_ms = timed(fp8.fp8_gemm_dscale, args.steps, args.warmup)
    value = flops / ms_step * 1e-9                      # TFLOP/s over the whole step
    gemm_tflops = flops / gemm_ms * 1e-9
    cast_bytes = 5.0 * (M * K + K * N)                  # amax reads 2 B, cast reads 2 B + writes 1 B per element
    out_bytes = M * N * (2 if out_name == "bf16" else 4)

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("gemm_" + args.workload, {}).get("total_bytes")
        except Exception:
            traffic = None

    result = {
        "metric": "FP8 GEMM TFLOP/s + quantize GB/s on 1 MI355X, as % of FP8 MFMA / HBM peak",
        "value": round(value, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp8 operands (E5M2 x E4M3)" if fmtA else "fp8 operands (E4M3 x E4M3)",
        "data": "synthetic",
        "config": {
            "workload": "%s: amax+scale+cast of A[%dx%d] and B[%dx%d] (bf16 -> FP8), FP8 GEMM fp32-accumulate, %s out"
                        % (args.workload, M, K, K, N, out_name),
            "M": M, "N": N, "K": K,
            "arithmetic": "FP8 bytes widened exactly to fp16 in registers, fp16 MFMA products, fp32 accumulation",
            "input_generation_s": round(t_gen, 1),
            "untimed_before_warmup": "1 step + %d GEMM launches (clock ramp after idle)" % CLOCK_RAMP_LAUNCHES,
        },
        "breakdown_ms": {"amax_scale_cast": round(cast_ms, 4), "gemm_epilogue": round(gemm_ms, 4)},
        "roofline": {
            "kernel": "gemm_fast_kernel (fp16-instruction mode)",
            "bound": "mfma", "achieved": round(gemm_tflops, 1), "peak": PEAK_FP16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(gemm_tflops / PEAK_FP16_TFLOPS, 4),
            "frac_of_fp8_peak": round(gemm_tflops / PEAK_FP8_TFLOPS, 4),
            "flops_per_launch": flops, "avg_launch_ms": round(gemm_ms, 4), "traffic": traffic,
        },
        "roofline_cast": {
            "kernels": "amax_vec_kernel + quantize_vec_kernel over A and B",
            "bound": "hbm", "achieved": round(cast_bytes / cast_ms * 1e-6, 1), "peak": PEAK_HBM_GBS,
            "unit": "GB/s", "frac": round(cast_bytes / cast_ms * 1e-6 / PEAK_HBM_GBS, 4),
            "bytes_per_step": cast_bytes,
        },
        "algorithmic_bytes_gemm": M * K + K * N + out_bytes,
    }

    if not args.no_extras:
        # the same step with the FP8 matrix-core instructions (weaker error bound, see include/fp8mm.h)
        ms8, _, gemm8_ms = timed(fp8.fp8_gemm_mfma8_dscale, max(3, args.steps // 2), 2)
        result["fp8_instruction_variant"] = {
            "entry_point": "fp8_gemm_mfma8_dscale", "ms_per_step": round(ms8, 4),
            "value": round(flops / ms8 * 1e-9, 2), "unit": "TFLOP/s",
            "roofline": {"bound": "mfma", "achieved": round(flops / gemm8_ms * 1e-9, 1), "peak": PEAK_FP8_TFLOPS,
                         "unit": "TFLOP/s", "frac": round(flops / gemm8_ms * 1e-9 / PEAK_FP8_TFLOPS, 4)},
            "note": "meets 2^-10 * sum|ab| (hardware adder window), not the 2^-20 bound of the default path",
        }
        # the step of a recipe that takes its factors from past maxima (single-pass cast + amax)
        hist = torch.ones((2, 4), device="cuda")
        def delayed_step():
            for t, q, i, f in ((dA, qA, 0, fmtA), (dB, qB, 1, fmtB)):
                fp8.fp8_scale_from_amax_history(hist[i], f, scale[i:i + 1])
                fp8.fp8_quantize_amax(t.view(-1), f, scale[i:i + 1], q.view(-1), hist[i, 0:1])
            fp8.fp8_gemm_dscale(qA, fmtA, scale[0:1], qB, fmtB, scale[1:2], C)
        for t, i in ((dA, 0), (dB, 1)):               # a history that holds the tensors' maxima
            fp8.fp8_amax(t, amax[i:i + 1])
            hist[i] = amax[i]
        n_d = max(3, args.steps // 2)
        ms_d = _event_ms(torch, delayed_step, n_d)
        result["delayed_scaling_step"] = {
            "entry_points": "fp8_scale_from_amax_history + fp8_quantize_amax (one pass over A and B) + fp8_gemm_dscale",
            "ms_per_step": round(ms_d, 4), "value": round(flops / ms_d * 1e-9, 2), "unit": "TFLOP/s",
        }
        result["gemm_variants"] = gemm_variants(fp8, torch, qA, qB, scale, fmtA, fmtB, M, N, K, out_dtype, flops, args)
        del dA, dB, qA, qB, C
        torch.cuda.empty_cache()
        result["quantize_only"] = quantize_only(fp8, synth, torch, np, args)

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(A_bits, B_bits, M, N, K, fmtA, fmtB, flops)

    print(json.dumps(result))


def _event_ms(torch, fn, iters, warm=2):
    """Average duration of fn over iters launches, from events on torch's current stream."""
    stream = torch.cuda.current_stream()
    for _ in range(warm):
        fn()
    e = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    torch.cuda.synchronize()
    for a, b in e:
        a.record(stream)
        fn()
        b.record(stream)
    torch.cuda.synchronize()
    return sum(a.elapsed_time(b) for a, b in e) / iters


def gemm_variants(fp8, torch, qA, qB, scale, fmtA, fmtB, M, N, K, out_dtype, flops, args):
    """The same product through the other entry points: operands given transposed (the storage orders
    of the dgrad / wgrad GEMMs of a linear layer), FP8 output with output scale and amax, per-channel
    factors.  TFLOP/s of the GEMM launch alone."""
    iters = max(3, args.steps // 4)
    out = {}
    qAt, qBt = qA.t().contiguous(), qB.t().contiguous()
    C = torch.empty((M, N), dtype=out_dtype, device="cuda")
    for tA, tB, a, b in ((0, 1, qA, qBt), (1, 0, qAt, qB), (1, 1, qAt, qBt)):
        for flags, mode in ((0, "fp16_instr"), (fp8.FP8_GEMM_MFMA8, "fp8_instr")):
            ms = _event_ms(torch, lambda: fp8.fp8_gemm_ex(a, fmtA, tA, b, fmtB, tB, C, scale[0:1], scale[1:2], flags), iters)
            out["gemm_ex_transA%d_transB%d_%s" % (tA, tB, mode)] = {"ms": round(ms, 4), "TFLOP/s": round(flops / ms * 1e-9, 1)}
    del qAt, qBt
    D = torch.empty((M, N), dtype=torch.uint8, device="cuda")
    amax = torch.zeros(1, device="cuda")
    sD = torch.ones(1, device="cuda")
    sAv = torch.ones(M, device="cuda") * scale[0]
    sBv = torch.ones(N, device="cuda") * scale[1]
    for flags, mode in ((0, "fp16_instr"), (fp8.FP8_GEMM_MFMA8, "fp8_instr")):
        ms = _event_ms(torch, lambda: fp8.fp8_gemm_fused(qA, fmtA, 0, qB, fmtB, 0, D, fp8.FP8_OUT_E4M3, scale[0:1], scale[1:2],
                                                         sD, amax, flags), iters)
        out["gemm_fused_e4m3_out_amax_%s" % mode] = {"ms": round(ms, 4), "TFLOP/s": round(flops / ms * 1e-9, 1)}
        ms = _event_ms(torch, lambda: fp8.fp8_gemm_fused(qA, fmtA, 0, qB, fmtB, 0, C, fp8.FP8_OUT_BF16 if C.dtype == torch.bfloat16 else fp8.FP8_OUT_F32,
                                                         sAv, sBv, None, None, flags), iters)
        out["gemm_fused_per_row_per_col_%s" % mode] = {"ms": round(ms, 4), "TFLOP/s": round(flops / ms * 1e-9, 1)}
    return out


def quantize_only(fp8, synth, torch, np, args):
    """2^28 bf16 elements with outliers: amax, then the cast to E4M3 and to E5M2 (config 2)."""
    n = 1 << 28
    h = synth.config2(n)
    x = torch.from_numpy(h.view(np.int16)).view(torch.bfloat16).cuda()
    q = torch.empty(n, dtype=torch.uint8, device="cuda")
    amax = torch.zeros(1, device="cuda")
    scale = torch.zeros(1, device="cuda")
    stream = torch.cuda.current_stream()
    out = {"elements": n}

    def t(fn, iters):
        for _ in range(3):
            fn()
        e = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        torch.cuda.synchronize()
        for a, b in e:
            a.record(stream)
            fn()
            b.record(stream)
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in e) / iters

    iters = max(5, args.steps)
    ms = t(lambda: fp8.fp8_amax(x, amax), iters)
    out["amax"] = {"us": round(ms * 1e3, 1), "GB/s": round(2.0 * n / ms * 1e-6, 1),
                   "frac_of_hbm_peak": round(2.0 * n / ms * 1e-6 / PEAK_HBM_GBS, 4)}
    for fmt, name in ((0, "cast_e4m3"), (1, "cast_e5m2")):
        fp8.fp8_scale_from_amax(amax, fmt, scale)
        ms = t(lambda: fp8.fp8_quantize_dscale(x, fmt, scale, q), iters)
        out[name] = {"us": round(ms * 1e3, 1), "GB/s": round(3.0 * n / ms * 1e-6, 1),
                     "frac_of_hbm_peak": round(3.0 * n / ms * 1e-6 / PEAK_HBM_GBS, 4)}

    # variants of the cast (algorithmic bytes per element: bf16 in, bytes out)
    def rate(name, ms, bytes_per_elem):
        out[name] = {"us": round(ms * 1e3, 1), "GB/s": round(bytes_per_elem * n / ms * 1e-6, 1),
                     "frac_of_hbm_peak": round(bytes_per_elem * n / ms * 1e-6 / PEAK_HBM_GBS, 4)}
    rate("cast_amax_single_pass_e4m3", t(lambda: fp8.fp8_quantize_amax(x, 0, scale, q, amax), iters), 3.0)
    rate("cast_stochastic_e4m3", t(lambda: fp8.fp8_quantize_sr(x, 0, scale, 1234, q), iters), 3.0)
    rows, cols = 1 << 14, 1 << 14
    xm, qm = x.view(rows, cols), q.view(rows, cols)
    qt = torch.empty((cols, rows), dtype=torch.uint8, device="cuda")
    rate("cast_transpose_e4m3_16384x16384_both_orders", t(lambda: fp8.fp8_quantize_transpose(xm, 0, scale, qm, qt), iters), 4.0)
    del qt
    ar, sr = torch.zeros(rows, device="cuda"), torch.ones(rows, device="cuda")
    rate("amax_rows_16384x16384", t(lambda: fp8.fp8_amax_rows(xm, ar), iters), 2.0)
    rate("cast_rows_e4m3_16384x16384", t(lambda: fp8.fp8_quantize_rows(xm, 0, sr, qm), iters), 3.0)
    return out


def cpu_baseline(A_bits, B_bits, M, N, K, fmtA, fmtB, flops):
    """The oracle, as it stands, timed on the host cores over a bounded sample of the same
    workload: amax+scale+cast of up to 2^27 elements of each operand, GEMM reference for 512
    output rows; the step time is extrapolated linearly to the full tensors."""
    import numpy as np

    import oracle
    n_s = 1 << 27
    rows = 512
    t0 = time.perf_counter()
    a_s, b_s = A_bits.reshape(-1)[:n_s], B_bits.reshape(-1)[:n_s]
    sA = oracle.scale_from_amax(oracle.amax(a_s), fmtA)
    qa = oracle.quantize(a_s, fmtA, sA)
    sB = oracle.scale_from_amax(oracle.amax(b_s), fmtB)
    qb = oracle.quantize(b_s, fmtB, sB)
    t_cast = time.perf_counter() - t0
    n_cast = a_s.size + b_s.size
    del qa, qb
    # GEMM rows need whole operands in FP8: quantise the `rows` rows of A and all of B once (untimed)
    Aq = oracle.quantize(A_bits[:rows], fmtA, sA)
    Bq = oracle.quantize(B_bits, fmtB, sB)
    t0 = time.perf_counter()
    oracle.gemm_rows(Aq, fmtA, Bq, fmtB, np.arange(rows))
    t_gemm = time.perf_counter() - t0
    full = t_cast * (M * K + K * N) / float(n_cast) + t_gemm * M / rows
    return {
        "value": round(flops / full * 1e-12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "amax+cast of %d elements (%.2f s) + fp64 reference GEMM of %d of %d output rows "
                  "(%.2f s), extrapolated linearly to one full step (%.0f s)" % (n_cast, t_cast, rows, M, t_gemm, full),
    }


if __name__ == "__main__":
    main()
