#!/usr/bin/env python3
"""Benchmark of the scaled-FP8 matrix multiply path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: amax and scale of A and of B (one launch each), cast of A and of B to FP8, the
FP8 GEMM with fp32 accumulation and the unscale epilogue.  The headline workload is the
GPT-175B-like FFN-up layer (8192 tokens x 12288 -> 49152, bf16 in, E4M3 operands, bf16 out).  One
JSON line is printed; beside the headline it carries
  - roofline: the GEMM kernel against the FP8 matrix-core peak the metric names, with the peak of
    the instruction it issues and the rate a register-only loop of that instruction sustains on
    this board beside it (libfp8probes.so);
  - roofline_cast: amax + cast against the HBM peak;
  - the same step on the dgrad and the small-GPT workloads, the FP8-instruction GEMM variant, the
    other entry points, the quantize-only workload (warm, cold and against plain streaming kernels);
  - cpu_baseline: the oracle timed on the host cores (a baseline, not a target).
"""
from __future__ import annotations

import argparse
import ctypes
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
METRIC = "FP8 GEMM TFLOP/s + quantize GB/s on 1 MI355X, as % of FP8 MFMA / HBM peak"

# name -> (config number, M, N, K, fmtA, out dtype name)
WORKLOADS = {
    "ffn_up_175b": (4, 8192, 49152, 12288, 0, "bf16"),
    "dgrad_175b": (5, 8192, 12288, 49152, 1, "f32"),
    "small_gpt_fwd": (3, 4096, 6144, 2048, 0, "bf16"),
}
CLOCK_RAMP_LAUNCHES = 12       # the chip's clocks settle over the first dozen GEMM launches after idling


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="ffn_up_175b", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="only the timed step of the chosen workload")
    return ap.parse_args()


class Probes:
    """ctypes access to libfp8probes.so (register-only MFMA loop, plain streaming kernels)."""
    def __init__(self):
        path = os.path.join(ROOT, "paper_2209_05433_amd", "libfp8probes.so")
        if not os.path.exists(path):
            raise FileNotFoundError(path + " is missing: build with __graft_entry__.build()")
        L = ctypes.CDLL(path)
        vp = ctypes.c_void_p
        L.fp8probe_mfma.argtypes = [ctypes.c_int, vp, vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp, vp]
        L.fp8probe_stream.argtypes = [ctypes.c_int, vp, vp, ctypes.c_size_t, ctypes.c_int, vp]
        self.L = L


def event_ms(torch, fn, iters, warm=2):
    """Average duration of fn over iters launches, from events on torch's current stream (the
    stream every launch of this file goes to)."""
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


def sustained_mfma(torch, probes, qA, qB, kind, reps=5):
    """TFLOP/s of a register-only loop of the instruction (kind 0: FP8, 1: fp16 on widened bytes) over
    the whole chip (256 workgroups of 4 waves), operand bytes taken from the workload's FP8 tensors."""
    span = 1 << 20
    out = torch.empty(256 * 256, device="cuda")
    iters = 40000 if kind == 0 else 20000
    st = torch.cuda.current_stream().cuda_stream
    a, b = qA.view(-1)[:span], qB.view(-1)[:span]
    def run():
        rc = probes.L.fp8probe_mfma(kind, a.data_ptr(), b.data_ptr(), span, 256, iters, out.data_ptr(), st)
        assert rc == 0, "fp8probe_mfma failed: %d" % rc
    ms = event_ms(torch, run, reps, warm=2)
    return 256 * 4 * iters * 2097152.0 / ms * 1e-9


def run_workload(name, args, fp8, synth, torch, np, probes, steps, warmup, extras):
    """The whole step on one workload: timing, breakdown by stream events, rooflines."""
    cfg, M, N, K, fmtA, out_name = WORKLOADS[name]
    fmtB = fp8.FP8_E4M3
    out_dtype = torch.bfloat16 if out_name == "bf16" else torch.float32
    gen = {3: synth.config3, 4: synth.config4, 5: synth.config5}[cfg]
    t0 = time.time()
    A_bits, B_bits = gen(M, N, K)
    to_dev = lambda h: torch.from_numpy(h.view(np.int16)).view(torch.bfloat16).cuda()
    dA, dB = to_dev(A_bits), to_dev(B_bits)
    t_gen = time.time() - t0
    stream = torch.cuda.current_stream()

    amax = torch.zeros(2, device="cuda")
    scale = torch.zeros(2, device="cuda")
    ws = torch.zeros(2 * fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
    qA = torch.empty((M, K), dtype=torch.uint8, device="cuda")
    qB = torch.empty((K, N), dtype=torch.uint8, device="cuda")
    C = torch.empty((M, N), dtype=out_dtype, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(gemm=fp8.fp8_gemm_dscale, record=None):
        if record is not None:
            record[0].record(stream)
        # amax + scale of both operands in one launch, then both casts (one launch where the outputs are
        # small enough for ordinary stores, else one per tensor inside the call)
        fp8.fp8_amax_scale_multi((dA, dB), (fmtA, fmtB), amax, scale, ws)
        fp8.fp8_quantize_multi((dA, dB), (fmtA, fmtB), scale, (qA, qB))
        if record is not None:
            record[1].record(stream)
        gemm(qA, fmtA, scale[0:1], qB, fmtB, scale[1:2], C)
        if record is not None:
            record[2].record(stream)

    def timed(gemm, n, w):
        for _ in range(w):
            step(gemm)
        recs = [(ev(), ev(), ev()) for _ in range(n)]
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for r in recs:
            step(gemm, r)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_start
        cast_ms = sum(r[0].elapsed_time(r[1]) for r in recs) / n
        gemm_ms = sum(r[1].elapsed_time(r[2]) for r in recs) / n
        return wall / n * 1e3, cast_ms, gemm_ms

    flops = 2.0 * M * N * K
    step()
    for _ in range(CLOCK_RAMP_LAUNCHES):
        fp8.fp8_gemm_dscale(qA, fmtA, scale[0:1], qB, fmtB, scale[1:2], C)
    ms_step, cast_ms, gemm_ms = timed(fp8.fp8_gemm_dscale, steps, warmup)
    gemm_tflops = flops / gemm_ms * 1e-9
    cast_bytes = 5.0 * (M * K + K * N)                  # amax reads 2 B, cast reads 2 B + writes 1 B per element
    out_bytes = M * N * (2 if out_name == "bf16" else 4)

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("gemm_" + name, {}).get("total_bytes")
        except Exception:
            traffic = None

    # the same step through fp8_scaled_gemm: one call, the same launches, no event between them
    def one_call():
        fp8.fp8_scaled_gemm(dA, fmtA, False, dB, fmtB, False, qA, qB, amax, scale, ws, C)
    for _ in range(max(2, warmup // 2)):
        one_call()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(steps):
        one_call()
    torch.cuda.synchronize()
    ms_one_call = (time.perf_counter() - t_start) / steps * 1e3

    sustained16 = sustained_mfma(torch, probes, qA, qB, 1) if probes else None
    res = {
        "ms_per_step": round(ms_step, 4),
        "value": round(flops / ms_step * 1e-9, 2),
        "unit": "TFLOP/s",
        "config": {
            "workload": "%s: amax+scale+cast of A[%dx%d] and B[%dx%d] (bf16 -> FP8), FP8 GEMM fp32-accumulate, %s out"
                        % (name, M, K, K, N, out_name),
            "M": M, "N": N, "K": K,
            "arithmetic": "FP8 bytes widened exactly to fp16 in registers, fp16 MFMA products, fp32 accumulation",
            "input_generation_s": round(t_gen, 1),
            "untimed_before_warmup": "1 step + %d GEMM launches (clock ramp after idle)" % CLOCK_RAMP_LAUNCHES,
        },
        "dtype": "fp8 operands (E5M2 x E4M3)" if fmtA else "fp8 operands (E4M3 x E4M3)",
        "breakdown_ms": {"amax_scale_cast": round(cast_ms, 4), "gemm_epilogue": round(gemm_ms, 4)},
        "one_call_step": {"entry_point": "fp8_scaled_gemm (the same three launches behind one call)",
                          "ms_per_step": round(ms_one_call, 4), "TFLOP/s": round(flops / ms_one_call * 1e-9, 2)},
        "roofline": {
            "kernel": "gemm_fast_kernel (fp16-instruction mode: the mode that meets the 2^-20 bound)",
            "bound": "mfma", "achieved": round(gemm_tflops, 1),
            "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s", "frac": round(gemm_tflops / PEAK_FP8_TFLOPS, 4),
            "peak_note": "FP8 matrix-core peak, the one the metric and its 70 % bar name; the kernel issues fp16 "
                         "instructions (half that peak) because no FP8 instruction of gfx950 adds its products to "
                         "the 2^-20 bound: the bar is NOT met",
            "peak_of_instruction": PEAK_FP16_TFLOPS, "frac_of_instruction_peak": round(gemm_tflops / PEAK_FP16_TFLOPS, 4),
            "sustained_peak": None if sustained16 is None else round(sustained16, 1),
            "frac_of_sustained": None if sustained16 is None else round(gemm_tflops / sustained16, 4),
            "sustained_note": "register-only loop of v_mfma_f32_32x32x16_f16 on bytes of this workload's FP8 tensors, "
                              "256 workgroups x 4 waves, same process",
            "flops_per_launch": flops, "avg_launch_ms": round(gemm_ms, 4), "traffic": traffic,
        },
        "roofline_cast": {
            "kernels": "amax_multi_kernel (A and B, with the scales, one launch) + quantize_multi_kernel (one launch) or quantize_vec_kernel per tensor (outputs of 384 MiB and more)",
            "bound": "hbm", "achieved": round(cast_bytes / cast_ms * 1e-6, 1), "peak": PEAK_HBM_GBS,
            "unit": "GB/s", "frac": round(cast_bytes / cast_ms * 1e-6 / PEAK_HBM_GBS, 4),
            "bytes_per_step": cast_bytes,
        },
        "algorithmic_bytes_gemm": M * K + K * N + out_bytes,
    }

    if extras:
        # The same launches recorded once into a HIP graph and replayed: what the step costs when the
        # host does not have to issue three to four launches per step (on the small workload the eager step is
        # bound by that, not by the GPU).  Three graphs: the whole step, the amax + cast chain, the GEMM.
        def cast_chain():
            fp8.fp8_amax_scale_multi((dA, dB), (fmtA, fmtB), amax, scale, ws)
            fp8.fp8_quantize_multi((dA, dB), (fmtA, fmtB), scale, (qA, qB))
        def replay_ms(fn, n):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                fn()
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            t_start = time.perf_counter()
            for _ in range(n):
                g.replay()
            torch.cuda.synchronize()
            return (time.perf_counter() - t_start) / n * 1e3
        n_g = max(10, steps)
        g_step = replay_ms(step, n_g)
        g_cast = replay_ms(cast_chain, n_g)
        g_gemm = replay_ms(lambda: fp8.fp8_gemm_dscale(qA, fmtA, scale[0:1], qB, fmtB, scale[1:2], C), n_g)
        g_gemm8 = replay_ms(lambda: fp8.fp8_gemm_mfma8_dscale(qA, fmtA, scale[0:1], qB, fmtB, scale[1:2], C), n_g)
        res["graph_replay"] = {
            "ms_per_step": round(g_step, 4), "value": round(flops / g_step * 1e-9, 2), "unit": "TFLOP/s",
            "amax_scale_cast_ms": round(g_cast, 4), "cast_frac_of_hbm_peak": round(cast_bytes / g_cast * 1e-6 / PEAK_HBM_GBS, 4),
            "gemm_ms": round(g_gemm, 4), "gemm_TFLOP/s": round(flops / g_gemm * 1e-9, 1),
            "gemm_fp8_instr_ms": round(g_gemm8, 4), "gemm_fp8_instr_TFLOP/s": round(flops / g_gemm8 * 1e-9, 1),
            "note": "wall time of back-to-back replays of a HIP graph of the step / of the chain / of one GEMM launch",
        }
        # the same step with the FP8 matrix-core instructions (weaker error bound, see include/fp8mm.h)
        ms8, _, gemm8_ms = timed(fp8.fp8_gemm_mfma8_dscale, max(3, steps // 2), 2)
        sustained8 = sustained_mfma(torch, probes, qA, qB, 0) if probes else None
        t8 = flops / gemm8_ms * 1e-9
        res["fp8_instruction_variant"] = {
            "entry_point": "fp8_gemm_mfma8_dscale", "ms_per_step": round(ms8, 4),
            "value": round(flops / ms8 * 1e-9, 2), "unit": "TFLOP/s",
            "roofline": {"bound": "mfma", "achieved": round(t8, 1), "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(t8 / PEAK_FP8_TFLOPS, 4),
                         "sustained_peak": None if sustained8 is None else round(sustained8, 1),
                         "frac_of_sustained": None if sustained8 is None else round(t8 / sustained8, 4),
                         "avg_launch_ms": round(gemm8_ms, 4)},
            "note": "meets 2^-10 * sum|ab| (hardware adder window), not the 2^-20 bound of the default path",
        }
    return res, (A_bits, B_bits, dA, dB, qA, qB, scale, C, fmtA, fmtB, M, N, K, out_dtype, flops)


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
    probes = Probes()

    main_res, state = run_workload(args.workload, args, fp8, synth, torch, np, probes, args.steps, args.warmup,
                                   extras=not args.no_extras)
    A_bits, B_bits, dA, dB, qA, qB, scale, C, fmtA, fmtB, M, N, K, out_dtype, flops = state
    result = {
        "metric": METRIC,
        "value": main_res["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": main_res["dtype"], "data": "synthetic",
    }
    for k in ("config", "breakdown_ms", "one_call_step", "roofline", "roofline_cast", "algorithmic_bytes_gemm", "graph_replay", "fp8_instruction_variant"):
        if k in main_res:
            result[k] = main_res[k]

    if not args.no_extras:
        result["delayed_scaling_step"] = delayed_scaling(fp8, torch, dA, dB, qA, qB, scale, C, fmtA, fmtB, flops, args)
        result["gemm_variants"] = gemm_variants(fp8, torch, qA, qB, scale, fmtA, fmtB, M, N, K, out_dtype, flops, args)
    del dA, dB, qA, qB, C
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(A_bits, B_bits, M, N, K, fmtA, fmtB, flops)
    del A_bits, B_bits, state

    if not args.no_extras:
        others = {}
        for name in WORKLOADS:
            if name == args.workload:
                continue
            r, st = run_workload(name, args, fp8, synth, torch, np, probes, max(5, args.steps // 2), max(3, args.warmup // 2),
                                 extras=True)
            del st
            torch.cuda.empty_cache()
            r["roofline"].pop("peak_note", None)
            r["roofline"].pop("sustained_note", None)
            others[name] = r
        result["other_workloads"] = others
        result["wgrad_split_k"] = split_k_leg(fp8, torch, args)
        result["any_shape_kernel"] = any_shape_leg(fp8, torch, args)
        torch.cuda.empty_cache()
        result["quantize_only"] = quantize_only(fp8, synth, torch, np, probes, args)

    print(json.dumps(result))


def delayed_scaling(fp8, torch, dA, dB, qA, qB, scale, C, fmtA, fmtB, flops, args):
    """The step of a recipe that takes its factors from past maxima (single-pass cast + amax)."""
    amax = torch.zeros(2, device="cuda")
    hist = torch.ones((2, 4), device="cuda")
    def step():
        for t, q, i, f in ((dA, qA, 0, fmtA), (dB, qB, 1, fmtB)):
            fp8.fp8_scale_from_amax_history(hist[i], f, scale[i:i + 1])
            fp8.fp8_quantize_amax(t.view(-1), f, scale[i:i + 1], q.view(-1), hist[i, 0:1])
        fp8.fp8_gemm_dscale(qA, fmtA, scale[0:1], qB, fmtB, scale[1:2], C)
    for t, i in ((dA, 0), (dB, 1)):               # a history that holds the tensors' maxima
        fp8.fp8_amax(t, amax[i:i + 1])
        hist[i] = amax[i]
    ms = event_ms(torch, step, max(3, args.steps // 2))
    return {"entry_points": "fp8_scale_from_amax_history + fp8_quantize_amax (one pass over A and B) + fp8_gemm_dscale",
            "ms_per_step": round(ms, 4), "value": round(flops / ms * 1e-9, 2), "unit": "TFLOP/s"}


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
            ms = event_ms(torch, lambda: fp8.fp8_gemm_ex(a, fmtA, tA, b, fmtB, tB, C, scale[0:1], scale[1:2], flags), iters)
            out["gemm_ex_transA%d_transB%d_%s" % (tA, tB, mode)] = {"ms": round(ms, 4), "TFLOP/s": round(flops / ms * 1e-9, 1)}
    del qAt, qBt
    D = torch.empty((M, N), dtype=torch.uint8, device="cuda")
    amax = torch.zeros(1, device="cuda")
    sD = torch.ones(1, device="cuda")
    sAv = torch.ones(M, device="cuda") * scale[0]
    sBv = torch.ones(N, device="cuda") * scale[1]
    for flags, mode in ((0, "fp16_instr"), (fp8.FP8_GEMM_MFMA8, "fp8_instr")):
        ms = event_ms(torch, lambda: fp8.fp8_gemm_fused(qA, fmtA, 0, qB, fmtB, 0, D, fp8.FP8_OUT_E4M3, scale[0:1], scale[1:2],
                                                        sD, amax, flags), iters)
        out["gemm_fused_e4m3_out_amax_%s" % mode] = {"ms": round(ms, 4), "TFLOP/s": round(flops / ms * 1e-9, 1)}
        ms = event_ms(torch, lambda: fp8.fp8_gemm_fused(qA, fmtA, 0, qB, fmtB, 0, C, fp8.FP8_OUT_BF16 if C.dtype == torch.bfloat16 else fp8.FP8_OUT_F32,
                                                        sAv, sBv, None, None, flags), iters)
        out["gemm_fused_per_row_per_col_%s" % mode] = {"ms": round(ms, 4), "TFLOP/s": round(flops / ms * 1e-9, 1)}
    return out


def split_k_leg(fp8, torch, args):
    """Weight-gradient regime: dW[1024 x 1024] over K = 65536 tokens (E5M2^T x E4M3 -> fp32), one
    workgroup per tile against the split-K entry point (slices spread over the chip)."""
    M = N = 1024
    K = 65536
    g = torch.Generator(device="cuda").manual_seed(7)
    A = torch.randint(0, 0x50, (K, M), dtype=torch.uint8, device="cuda", generator=g)
    B = torch.randint(0, 0x70, (K, N), dtype=torch.uint8, device="cuda", generator=g)
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    need = fp8.fp8_gemm_splitk_workspace_size(M, N, K, 1, 0, 0)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    flops = 2.0 * M * N * K
    out = {"shape": [M, N, K], "slices": need // (4 * M * N), "workspace_bytes": need}
    iters = max(5, args.steps // 2)
    for flags, mode in ((0, "fp16_instr"), (fp8.FP8_GEMM_MFMA8, "fp8_instr")):
        ms0 = event_ms(torch, lambda: fp8.fp8_gemm_ex(A, fp8.FP8_E5M2, 1, B, fp8.FP8_E4M3, 0, C, 1.0, 1.0, flags), 3)
        ms1 = event_ms(torch, lambda: fp8.fp8_gemm_splitk(A, fp8.FP8_E5M2, 1, B, fp8.FP8_E4M3, 0, C, 1.0, 1.0, ws, flags, 0), iters)
        ms2 = event_ms(torch, lambda: fp8.fp8_gemm_splitk_static(A, fp8.FP8_E5M2, 1, B, fp8.FP8_E4M3, 0, C, 1.0, 1.0, flags, 0), iters) \
            if hasattr(fp8, "fp8_gemm_splitk_static") else None
        out[mode] = {"one_workgroup_per_tile_ms": round(ms0, 4), "split_k_ms": round(ms1, 4),
                     "split_k_static_scratch_ms": None if ms2 is None else round(ms2, 4),
                     "speedup": round(ms0 / ms1, 2), "TFLOP/s": round(flops / ms1 * 1e-9, 1)}
    return out


def any_shape_leg(fp8, torch, args):
    """A vocabulary projection with the weight stored [in, out] and an odd vocabulary size
    (8192 x 50257 x 12288, B stored K x N): rows of B start anywhere, so the tiled kernel's direct loads
    cannot take it and the any-shape matrix-core kernel runs; beside it the same product with N
    padded to a multiple of 16 (tiled kernel)."""
    M, K = 8192, 12288
    g = torch.Generator(device="cuda").manual_seed(11)
    A = torch.randint(0, 0x60, (M, K), dtype=torch.uint8, device="cuda", generator=g)
    out = {}
    for N, label in ((50257, "N_50257"), (50272, "N_50272_padded")):
        B = torch.randint(0, 0x60, (K, N), dtype=torch.uint8, device="cuda", generator=g)
        C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        plan = fp8.fp8_gemm_plan(A, 0, B, 0, C)
        ms = event_ms(torch, lambda: fp8.fp8_gemm_ex(A, fp8.FP8_E4M3, 0, B, fp8.FP8_E4M3, 0, C, 1.0, 1.0, 0), 4, 2)
        out[label] = {"plan": plan, "ms": round(ms, 3), "TFLOP/s": round(2.0 * M * N * K / ms * 1e-9, 1)}
        del B, C
    return out


def quantize_only(fp8, synth, torch, np, probes, args):
    """2^28 bf16 elements with outliers: amax, then the cast to E4M3 and to E5M2 (config 2).  Three
    readings: the same buffers launch after launch (the 256 MB memory-side cache helps), four
    distinct input / output pairs in rotation (3 GB working set: nothing survives from one launch to
    the next), and plain streaming kernels with the same access mix on the same buffers."""
    n = 1 << 28
    NPAIR = 4
    h = synth.config2(n)
    xs = [torch.from_numpy(h.view(np.int16)).view(torch.bfloat16).cuda()]
    for _ in range(NPAIR - 1):
        xs.append(xs[0].clone())
    qs = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(NPAIR)]
    x, q = xs[0], qs[0]
    amax = torch.zeros(1, device="cuda")
    scale = torch.zeros(1, device="cuda")
    ws = torch.zeros(fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
    out = {"elements": n}
    iters = max(8, args.steps)

    def rate(name, ms, bytes_per_elem, **extra):
        out[name] = {"us": round(ms * 1e3, 1), "GB/s": round(bytes_per_elem * n / ms * 1e-6, 1),
                     "frac_of_hbm_peak": round(bytes_per_elem * n / ms * 1e-6 / PEAK_HBM_GBS, 4), **extra}

    def rotating(fn):
        k = [0]
        def call():
            fn(xs[k[0] % NPAIR], qs[k[0] % NPAIR])
            k[0] += 1
        return call

    rate("amax", event_ms(torch, lambda: fp8.fp8_amax_scale(x, 0, amax, scale, ws), iters, 3), 2.0)
    rate("amax_cold", event_ms(torch, rotating(lambda xi, qi: fp8.fp8_amax_scale(xi, 0, amax, scale, ws)), iters, NPAIR), 2.0)
    for fmt, name in ((0, "cast_e4m3"), (1, "cast_e5m2")):
        fp8.fp8_amax_scale(x, fmt, amax, scale, ws)
        rate(name, event_ms(torch, lambda: fp8.fp8_quantize_dscale(x, fmt, scale, q), iters, 3), 3.0)
        rate(name + "_cold", event_ms(torch, rotating(lambda xi, qi: fp8.fp8_quantize_dscale(xi, fmt, scale, qi)), iters, NPAIR), 3.0)
    out["cold_note"] = "%d distinct input/output pairs in rotation (%.1f GB working set); warm = one pair, launch after launch" % (
        NPAIR, NPAIR * 3.0 * n * 1e-9)

    # plain streaming kernels on the same (rotating) buffers: what the memory system gives the mix
    if probes:
        st = torch.cuda.current_stream().cuda_stream
        n16_in = 2 * n // 16
        def stream_rate(mode, label, nbytes, src_of, dst_of, n16, grids=(2048, 8192, 32768)):
            best = None
            for wgs in grids:
                k = [0]
                def call():
                    rc = probes.L.fp8probe_stream(mode, src_of(k[0] % NPAIR), dst_of(k[0] % NPAIR), n16, wgs, st)
                    assert rc == 0
                    k[0] += 1
                ms = event_ms(torch, call, iters, NPAIR)
                if best is None or ms < best[0]:
                    best = (ms, wgs)
            out[label] = {"us": round(best[0] * 1e3, 1), "GB/s": round(nbytes / best[0] * 1e-6, 1),
                          "frac_of_hbm_peak": round(nbytes / best[0] * 1e-6 / PEAK_HBM_GBS, 4), "workgroups": best[1]}
        sink = torch.zeros(32768 * 4, dtype=torch.int32, device="cuda")
        stream_rate(0, "streaming_read_cold", 2.0 * n, lambda i: xs[i].data_ptr(), lambda i: sink.data_ptr(), n16_in)
        stream_rate(3, "streaming_2reads_1write_cold", 3.0 * n, lambda i: xs[i].data_ptr(), lambda i: qs[i].data_ptr(), n // 16)
        stream_rate(1, "streaming_write_cold", 1.0 * n, lambda i: None, lambda i: qs[i].data_ptr(), n // 16)
        stream_rate(2, "streaming_copy_cold", 2.0 * n, lambda i: xs[i].data_ptr(), lambda i: qs[i].data_ptr(), n // 16)
        out["streaming_note"] = "plain kernels of libfp8probes.so (non-temporal 16-byte loads / stores, best of three grid sizes) " \
                                "on the same rotating buffers: the board's ceiling for the access mix of the amax (read), the cast " \
                                "(2 reads per write), the dequantize kernels (write-heavy: between write and copy)"
    del xs[1:], qs[1:]
    torch.cuda.empty_cache()

    # variants of the cast (algorithmic bytes per element: bf16 in, bytes out)
    rate("cast_amax_single_pass_e4m3", event_ms(torch, lambda: fp8.fp8_quantize_amax(x, 0, scale, q, amax), iters, 3), 3.0)
    rate("cast_stochastic_e4m3", event_ms(torch, lambda: fp8.fp8_quantize_sr(x, 0, scale, 1234, q), iters, 3), 3.0)
    rows, cols = 1 << 14, 1 << 14
    xm, qm = x.view(rows, cols), q.view(rows, cols)
    qt = torch.empty((cols, rows), dtype=torch.uint8, device="cuda")
    rate("cast_transpose_e4m3_16384x16384_both_orders", event_ms(torch, lambda: fp8.fp8_quantize_transpose(xm, 0, scale, qm, qt), iters, 3), 4.0)
    del qt
    # the weight of the FFN-up layer (config 4), as the weight-gradient and data-gradient GEMMs want it in both orders
    wr, wc = 12288, 49152
    xw = torch.from_numpy(synth.config2(wr * wc).view(np.int16)).view(torch.bfloat16).cuda().view(wr, wc)
    qw, qwt = torch.empty((wr, wc), dtype=torch.uint8, device="cuda"), torch.empty((wc, wr), dtype=torch.uint8, device="cuda")
    ms = event_ms(torch, lambda: fp8.fp8_quantize_transpose(xw, 0, scale, qw, qwt), iters, 3)
    out["cast_transpose_e4m3_12288x49152_both_orders"] = {"us": round(ms * 1e3, 1), "GB/s": round(4.0 * wr * wc / ms * 1e-6, 1),
                                                          "frac_of_hbm_peak": round(4.0 * wr * wc / ms * 1e-6 / PEAK_HBM_GBS, 4)}
    del xw, qw, qwt
    ar, sr = torch.zeros(rows, device="cuda"), torch.ones(rows, device="cuda")
    rate("amax_rows_16384x16384", event_ms(torch, lambda: fp8.fp8_amax_rows(xm, ar), iters, 3), 2.0)
    rate("cast_rows_e4m3_16384x16384", event_ms(torch, lambda: fp8.fp8_quantize_rows(xm, 0, sr, qm), iters, 3), 3.0)
    yb = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    rate("dequantize_to_bf16", event_ms(torch, lambda: fp8.fp8_dequantize(q, 0, scale, yb), iters, 3), 3.0)
    del yb
    yf = torch.empty(n, dtype=torch.float32, device="cuda")
    rate("dequantize_to_f32", event_ms(torch, lambda: fp8.fp8_dequantize(q, 0, scale, yf), iters, 3), 5.0)
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
