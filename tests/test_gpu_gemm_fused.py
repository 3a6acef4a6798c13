"""GPU parity: fp8_gemm_fused (per-channel scaling factors, FP8 outputs with an output scale, output
amax) against the CPU oracle.

Acceptance.  c_ij = S_ij / (sA_i sB_j) is held to the GEMM bound
    |c_gpu - c_ref| <= rel * T_ij / (sA_i sB_j) (+ ulp_out / 2 for fp32 / bf16 outputs),
rel = 2^-20 (2^-10 with the FP8 matrix-core instructions).  An FP8 output byte is a rounding
decision taken on the kernel's own c: it must be the encoding of some value within that bound of
c_ref * sD, i.e. lie between encode(c_ref * sD - b) and encode(c_ref * sD + b) in value order; where
the sums are exact in fp32 it must be the oracle's byte.  amax_out must lie between
max(|c_ref| - b) and max(|c_ref| + b)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2209_05433_amd as fp8
from workloads import synth
from gpu_util import to_dev, out_to_f64, knob
from test_gpu_gemm import random_codes, sample_points, REL, MODES

pytestmark = pytest.mark.gpu

E4M3, E5M2 = fp8.FP8_E4M3, fp8.FP8_E5M2
OUT_T = {fp8.FP8_OUT_F32: torch.float32, fp8.FP8_OUT_BF16: torch.bfloat16,
         fp8.FP8_OUT_E4M3: torch.uint8, fp8.FP8_OUT_E5M2: torch.uint8}
FMT_OF = {fp8.FP8_OUT_E4M3: E4M3, fp8.FP8_OUT_E5M2: E5M2}
FMT_MAX = {E4M3: 448.0, E5M2: 57344.0}


def flags_of(mode):
    return fp8.FP8_GEMM_MFMA8 if mode == "mfma8" else 0


def dev_f32(v):
    return torch.from_numpy(np.atleast_1d(np.asarray(v, dtype=np.float32))).cuda()


def run_fused(A, fmtA, B, fmtB, out_kind, sA, sB, sD=None, want_amax=False, mode="f16", transA=0, transB=0):
    """A is M x K, B is K x N on the host (transposed copies are made for the device if asked)."""
    dA = to_dev(np.ascontiguousarray(A.T) if transA else A)
    dB = to_dev(np.ascontiguousarray(B.T) if transB else B)
    D = torch.empty((A.shape[0], B.shape[1]), dtype=OUT_T[out_kind], device="cuda")
    D.fill_(0x55 if D.dtype == torch.uint8 else 12345.0)
    amax = torch.full((1,), -1.0, device="cuda") if want_amax else None
    fp8.fp8_gemm_fused(dA, fmtA, transA, dB, fmtB, transB, D, out_kind, dev_f32(sA), dev_f32(sB),
                       None if sD is None else dev_f32(sD), amax, flags_of(mode))
    torch.cuda.synchronize()
    return D, (None if amax is None else np.float32(amax.item()))


def reference(S, T, sA, sB, mode):
    if np.size(sA) == 1 and np.size(sB) == 1:
        c_ref, alpha = oracle.unscale(S, np.float32(sA).reshape(()), np.float32(sB).reshape(()))
    else:
        c_ref, alpha = oracle.unscale_channels(S, sA, sB)
    return c_ref, REL[mode] * alpha * np.abs(T)


def check_wide(D, S, T, sA, sB, out_kind, mode, what):
    c_ref, b = reference(S, T, sA, sB, mode)
    bound = b + 0.5 * oracle.ulp(c_ref, out_kind)
    err = np.abs(out_to_f64(D) - c_ref)
    assert np.all(err <= bound), "%s: worst err/bound %.3g" % (what, np.max(err / bound))


def check_fp8_bytes(got, c_ref, b, sD, fmt, what, min_exact=0.97):
    """got: uint8 array.  Every byte must encode a value within the bound of c_ref * sD."""
    dec = oracle.decode_all(fmt)
    y = c_ref * float(sD)
    by = b * float(sD) + np.abs(y) * 2.0 ** -22          # + the fp32 roundings of c * sD
    lo = oracle.quantize((y - by).astype(np.float32), fmt, 1.0)
    hi = oracle.quantize((y + by).astype(np.float32), fmt, 1.0)
    v, vlo, vhi = dec[got], dec[lo], dec[hi]
    ok = (v >= vlo) & (v <= vhi)
    assert np.all(ok), "%s: %d of %d bytes outside the admissible range; first at %s: got 0x%02x, range 0x%02x..0x%02x" % (
        what, np.count_nonzero(~ok), ok.size, np.argwhere(~ok)[0], got[~ok][0], lo[~ok][0], hi[~ok][0])
    want = oracle.quantize(y.astype(np.float32), fmt, 1.0)
    exact = np.mean(got == want)
    assert exact >= min_exact, "%s: only %.4f of the bytes equal the oracle's" % (what, exact)
    return exact


def check_amax(amax, c_ref, b, what):
    lo, hi = np.max(np.abs(c_ref) - b), np.max(np.abs(c_ref) + b)
    assert lo * (1 - 2.0 ** -22) <= float(amax) <= hi * (1 + 2.0 ** -22), "%s: amax %r outside [%r, %r]" % (what, amax, lo, hi)


def int_codes(rng, shape):
    """E4M3 codes of integers in [-4, 4]: every partial sum of products is an integer below 2^24,
    so fp32 accumulation is exact in any order."""
    return oracle.quantize(rng.integers(-4, 5, shape).astype(np.float32), E4M3, 1.0)


SHAPES = [(512, 256, 640), (100, 36, 72)]          # tiled kernel (several tiles), generic kernel (ragged)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("a_vec,b_vec", [(1, 0), (0, 1), (1, 1), (0, 0)])
def test_per_channel_scales(a_vec, b_vec, mode):
    rng = np.random.default_rng(100 + 2 * a_vec + b_vec)
    for (M, N, K) in SHAPES:
        A = random_codes(rng, (M, K), E4M3)
        B = random_codes(rng, (K, N), E4M3)
        S, T = oracle.gemm_rows(A, E4M3, B, E4M3)
        sA = (rng.uniform(0.5, 300.0, M) if a_vec else rng.uniform(0.5, 300.0, 1)).astype(np.float32)
        sB = (2.0 ** rng.uniform(-8, 8, N) if b_vec else rng.uniform(0.01, 2.0, 1)).astype(np.float32)
        for out_kind in (fp8.FP8_OUT_F32, fp8.FP8_OUT_BF16):
            for (tA, tB) in ((0, 0), (1, 1)):
                D, _ = run_fused(A, E4M3, B, E4M3, out_kind, sA, sB, mode=mode, transA=tA, transB=tB)
                check_wide(D, S, T, sA, sB, out_kind, mode, "per-channel %s a_vec=%d b_vec=%d out=%d layout %d%d" % (
                    (M, N, K), a_vec, b_vec, out_kind, tA, tB))


def test_per_channel_scales_are_not_swapped_or_shifted():
    """Integer operands (exact sums) and power-of-two factors that differ in every row and column:
    the result is exact, so any mix-up of a row or column index shows as a mismatch."""
    rng = np.random.default_rng(7)
    for (M, N, K) in SHAPES:
        A, B = int_codes(rng, (M, K)), int_codes(rng, (K, N))
        S, T = oracle.gemm_rows(A, E4M3, B, E4M3)
        sA = np.ldexp(1.0, (np.arange(M) * 7) % 13 - 6).astype(np.float32)
        sB = np.ldexp(1.0, (np.arange(N) * 5) % 11 - 5).astype(np.float32)
        c_ref, _ = oracle.unscale_channels(S, sA, sB)
        for mode in MODES:
            D, amax = run_fused(A, E4M3, B, E4M3, fp8.FP8_OUT_F32, sA, sB, want_amax=True, mode=mode)
            assert np.array_equal(out_to_f64(D), c_ref), (M, N, K, mode)
            assert float(amax) == np.max(np.abs(c_ref))


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("out_kind", [fp8.FP8_OUT_E4M3, fp8.FP8_OUT_E5M2])
def test_fp8_output_with_output_scale_and_amax(out_kind, mode):
    fmt = FMT_OF[out_kind]
    rng = np.random.default_rng(200 + out_kind)
    for (M, N, K) in SHAPES:
        A = random_codes(rng, (M, K), E4M3, 0x6F)
        B = random_codes(rng, (K, N), E4M3, 0x6F)
        S, T = oracle.gemm_rows(A, E4M3, B, E4M3)
        sA, sB = np.float32(3.0), np.float32(0.7)
        c_ref, b = reference(S, T, sA, sB, mode)
        amax_ref = np.max(np.abs(c_ref))
        for sD in (np.float32(FMT_MAX[fmt] / amax_ref), np.float32(8 * FMT_MAX[fmt] / amax_ref), np.float32(1e-3)):
            # 8x too large a factor: the largest outputs saturate; a tiny one: subnormals and zeros
            D, amax = run_fused(A, E4M3, B, E4M3, out_kind, sA, sB, sD=sD, want_amax=True, mode=mode)
            got = D.cpu().numpy()
            check_fp8_bytes(got, c_ref, b, sD, fmt, "fp8 out %s fmt %d sD %g %s" % ((M, N, K), fmt, sD, mode),
                            min_exact=0.999 if mode == "f16" else 0.80)
            assert not np.any((got & 0x7F) > (0x7E if fmt == E4M3 else 0x7B)), "non-finite byte from finite data"
            check_amax(amax, c_ref, b, "fp8 out amax")
        # per-channel factors together with an FP8 output, transposed operands
        sAv = rng.uniform(0.5, 4.0, M).astype(np.float32)
        sBv = rng.uniform(0.5, 4.0, N).astype(np.float32)
        c_ref, b = reference(S, T, sAv, sBv, mode)
        sD = np.float32(FMT_MAX[fmt] / np.max(np.abs(c_ref)))
        D, amax = run_fused(A, E4M3, B, E4M3, out_kind, sAv, sBv, sD=sD, want_amax=True, mode=mode, transA=1, transB=1)
        check_fp8_bytes(D.cpu().numpy(), c_ref, b, sD, fmt, "fp8 out, per-channel", min_exact=0.999 if mode == "f16" else 0.80)
        check_amax(amax, c_ref, b, "fp8 out amax, per-channel")


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("out_kind", [fp8.FP8_OUT_E4M3, fp8.FP8_OUT_E5M2])
def test_fp8_output_is_the_oracle_byte_where_sums_are_exact(out_kind, mode):
    """Small-integer operands: every dot product is exact in fp32, so c is the exact value and the
    output byte must be the oracle's, ties included (integers hit many FP8 midpoints)."""
    fmt = FMT_OF[out_kind]
    rng = np.random.default_rng(300 + out_kind)
    for (M, N, K) in SHAPES:
        A, B = int_codes(rng, (M, K)), int_codes(rng, (K, N))
        S, _ = oracle.gemm_rows(A, E4M3, B, E4M3)
        for sD in (np.float32(1.0), np.float32(2.0 ** -3), np.float32(64.0)):
            D, amax = run_fused(A, E4M3, B, E4M3, out_kind, np.float32(2.0), np.float32(0.25), sD=sD,
                                want_amax=True, mode=mode)
            c_ref = S / 0.5
            want = oracle.quantize((c_ref * float(sD)).astype(np.float32), fmt, 1.0)
            got = D.cpu().numpy()
            assert np.array_equal(got, want), "%s sD %g: %d bytes differ" % ((M, N, K), sD, np.count_nonzero(got != want))
            assert float(amax) == np.max(np.abs(c_ref))
        # without an output scale pointer the factor is 1
        D, _ = run_fused(A, E4M3, B, E4M3, out_kind, np.float32(2.0), np.float32(0.25), mode=mode)
        assert np.array_equal(D.cpu().numpy(), oracle.quantize((S / 0.5).astype(np.float32), fmt, 1.0))


@pytest.mark.parametrize("mode", MODES)
def test_fp8_output_special_values_and_amax_nan(mode):
    """inf and NaN accumulators: E4M3 output has no infinity (inf -> NaN), E5M2 keeps it; amax
    reports NaN if any output is NaN, else +inf (Section 2, conversion of special values)."""
    for (M, N, K) in SHAPES:
        A = np.full((M, K), 0x38, np.uint8)      # 1.0 (E5M2: 0x3C)
        A[:] = 0x3C
        B = np.full((K, N), 0x38, np.uint8)      # 1.0 in E4M3
        A[1, 0] = 0x7C                           # +inf in E5M2  -> row 1 = +inf
        A[2, 3] = 0xFC                           # -inf          -> row 2 = -inf
        for with_nan in (False, True):
            if with_nan:
                A[M - 1, K - 1] = 0x7E           # NaN           -> last row = NaN
            for out_kind, fmt in ((fp8.FP8_OUT_E4M3, E4M3), (fp8.FP8_OUT_E5M2, E5M2)):
                D, amax = run_fused(A, E5M2, B, E4M3, out_kind, np.float32(1.0), np.float32(1.0), sD=np.float32(0.5),
                                    want_amax=True, mode=mode)
                got = D.cpu().numpy()
                if fmt == E4M3:
                    assert np.all((got[1] & 0x7F) == 0x7F) and np.all((got[2] & 0x7F) == 0x7F)
                else:
                    assert np.all(got[1] == 0x7C) and np.all(got[2] == 0xFC)
                finite_rows = [0, 3, M - 2]
                want = oracle.quantize(np.full(N, K * 0.5, np.float32), fmt, 1.0)
                for r in finite_rows:
                    assert np.array_equal(got[r], want)
                if with_nan:
                    nan_codes = (got[M - 1] & 0x7F)
                    assert np.all(nan_codes == 0x7F) if fmt == E4M3 else np.all(nan_codes > 0x7C)
                    assert np.isnan(amax)
                else:
                    assert amax == np.inf


def test_amax_out_with_wide_outputs_and_degenerate_shapes():
    rng = np.random.default_rng(11)
    M, N, K = 256, 256, 128
    A = random_codes(rng, (M, K), E4M3)
    B = random_codes(rng, (K, N), E4M3)
    S, T = oracle.gemm_rows(A, E4M3, B, E4M3)
    for mode in MODES:
        c_ref, b = reference(S, T, np.float32(1.5), np.float32(1.5), mode)
        for out_kind in (fp8.FP8_OUT_F32, fp8.FP8_OUT_BF16):
            D, amax = run_fused(A, E4M3, B, E4M3, out_kind, np.float32(1.5), np.float32(1.5), want_amax=True, mode=mode)
            check_amax(amax, c_ref, b, "amax, wide output")
            check_wide(D, S, T, np.float32(1.5), np.float32(1.5), out_kind, mode, "wide output with amax")
    # K = 0: all outputs are +0 (byte 0x00), amax 0; M = 0: nothing written, amax 0
    D, amax = run_fused(A[:, :0], E4M3, B[:0, :], E4M3, fp8.FP8_OUT_E4M3, np.float32(1.0), np.float32(1.0), want_amax=True)
    assert not D.cpu().numpy().any() and amax == 0.0
    D, amax = run_fused(A[:0], E4M3, B, E4M3, fp8.FP8_OUT_E5M2, np.float32(1.0), np.float32(1.0), want_amax=True)
    assert amax == 0.0


def test_fused_rejects_bad_arguments():
    A = torch.zeros((256, 128), dtype=torch.uint8, device="cuda")
    B = torch.zeros((128, 256), dtype=torch.uint8, device="cuda")
    D = torch.zeros((256, 256), dtype=torch.uint8, device="cuda")
    one = torch.ones(1, device="cuda")
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_gemm_fused(A, E4M3, 0, B, E4M3, 0, D, fp8.FP8_OUT_E4M3, torch.ones(7, device="cuda"), one)
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_gemm_fused(A, E4M3, 0, B, E4M3, 0, D, fp8.FP8_OUT_E4M3, one, torch.ones(255, device="cuda"))
    Df = torch.zeros((256, 256), dtype=torch.float32, device="cuda")
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_gemm_fused(A, E4M3, 0, B, E4M3, 0, Df, fp8.FP8_OUT_F32, one, one, sD=one)
    assert not D.cpu().numpy().any()


def test_config4_shape_fp8_output_full_size():
    """FFN-up shape at full size (M 8192, N 49152, K 12288): E4M3 output with the output scale taken
    from a first pass's amax (the two-pass form of current scaling), checked at sampled points."""
    A_bits, B_bits = synth.config4()
    fmtA = fmtB = E4M3
    sA = oracle.scale_from_amax(oracle.amax(A_bits), fmtA)
    sB = oracle.scale_from_amax(oracle.amax(B_bits), fmtB)
    Aq, Bq = oracle.quantize(A_bits, fmtA, sA), oracle.quantize(B_bits, fmtB, sB)
    del A_bits, B_bits
    M, K = Aq.shape
    N = Bq.shape[1]
    dA, dB = to_dev(Aq), to_dev(Bq)
    dsA, dsB = dev_f32(sA), dev_f32(sB)
    amax = torch.zeros(1, device="cuda")
    sD = torch.zeros(1, device="cuda")
    C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    D = torch.empty((M, N), dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(4)
    pi, pj = sample_points(rng, M, N, 3000)
    S, T = oracle.gemm_points(Aq, fmtA, Bq, fmtB, pi, pj)
    ti, tj = torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda()
    for mode in MODES:
        fp8.fp8_gemm_fused(dA, fmtA, 0, dB, fmtB, 0, C, fp8.FP8_OUT_BF16, dsA, dsB, None, amax, flags_of(mode))
        fp8.fp8_scale_from_amax(amax, E4M3, sD)
        fp8.fp8_gemm_fused(dA, fmtA, 0, dB, fmtB, 0, D, fp8.FP8_OUT_E4M3, dsA, dsB, sD, None, flags_of(mode))
        torch.cuda.synchronize()
        c_ref, b = reference(S, T, sA, sB, mode)
        # amax over the whole matrix: at least what the sampled points show, and equal to the max of
        # the bf16 outputs up to their rounding
        a = float(amax.item())
        assert a >= np.max(np.abs(c_ref) - b)
        cmax = float(C.float().abs().max().item())
        assert abs(a - cmax) <= a * 2.0 ** -8
        assert np.float32(sD.item()) == oracle.scale_from_amax(np.float32(a), E4M3)
        exact = check_fp8_bytes(D[ti, tj].cpu().numpy(), c_ref, b, np.float32(sD.item()), E4M3, "config 4 fp8 out " + mode,
                                min_exact=0.999 if mode == "f16" else 0.80)
        check_wide(C[ti, tj], S, T, sA, sB, fp8.FP8_OUT_BF16, mode, "config 4 bf16 out via fused " + mode)
        print("config 4 shape, E4M3 output (%s): %.4f of sampled bytes equal the oracle's" % (mode, exact), flush=True)


RAGGED = [(300, 272, 256), (8, 16, 128), (1, 1008, 384), (1000, 48, 128), (513, 528, 256), (255, 256, 128)]


@pytest.fixture(params=["256", "128"])
def tile_n(request):
    """Both tile widths of the tiled kernel, whatever the dispatcher would choose."""
    import os
    old = fp8.fp8_set_knob(fp8.FP8_KNOB_TILE_N, int(request.param))
    yield request.param
    fp8.fp8_set_knob(fp8.FP8_KNOB_TILE_N, old)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_edge_tiles_of_the_tiled_kernel(transA, transB, mode, tile_n):
    """M and N that are not multiples of the 256 x 256 tile (N a multiple of 16, M too if A is stored
    K x M) run in the tiled kernel with clipped edge tiles: every output kind, per-channel factors
    and the output amax must come out as for whole tiles, and nothing may be written past the edges."""
    rng = np.random.default_rng(400 + 2 * transA + transB)
    for (M, N, K) in RAGGED:
        if transA and M % 16:
            M = (M + 15) // 16 * 16
        A = random_codes(rng, (M, K), E4M3)
        B = random_codes(rng, (K, N), E5M2, 0x6F)
        S, T = oracle.gemm_rows(A, E4M3, B, E5M2)
        sA = rng.uniform(0.5, 4.0, M).astype(np.float32)
        sB = rng.uniform(0.5, 4.0, N).astype(np.float32)
        dA = to_dev(np.ascontiguousarray(A.T) if transA else A)
        dB = to_dev(np.ascontiguousarray(B.T) if transB else B)
        c_ref, b = reference(S, T, sA, sB, mode)
        for out_kind in (fp8.FP8_OUT_F32, fp8.FP8_OUT_BF16, fp8.FP8_OUT_E4M3):
            # the output sits inside a larger buffer whose surroundings must stay untouched
            esz = {fp8.FP8_OUT_F32: 4, fp8.FP8_OUT_BF16: 2, fp8.FP8_OUT_E4M3: 1}[out_kind]
            pad = 4096 // esz
            buf = torch.zeros(2 * pad + M * N, dtype=OUT_T[out_kind], device="cuda")
            buf.fill_(7)
            D = buf[pad:pad + M * N].view(M, N)
            amax = torch.full((1,), -1.0, device="cuda")
            sD = None
            if out_kind == fp8.FP8_OUT_E4M3:
                sD = dev_f32(np.float32(448.0 / np.max(np.abs(c_ref))))
            fp8.fp8_gemm_fused(dA, E4M3, transA, dB, E5M2, transB, D, out_kind, dev_f32(sA), dev_f32(sB), sD, amax,
                               flags_of(mode))
            torch.cuda.synchronize()
            what = "edge tiles %s layout %d%d out %d %s" % ((M, N, K), transA, transB, out_kind, mode)
            assert bool((buf[:pad] == 7).all()) and bool((buf[pad + M * N:] == 7).all()), what + ": wrote outside D"
            if out_kind == fp8.FP8_OUT_E4M3:
                check_fp8_bytes(D.cpu().numpy(), c_ref, b, np.float32(sD.item()), E4M3, what,
                                min_exact=0.99 if mode == "f16" else 0.80)
            else:
                check_wide(D, S, T, sA, sB, out_kind, mode, what)
            check_amax(np.float32(amax.item()), c_ref, b, what)


def test_edge_tiles_agree_with_the_generic_kernel_exactly_on_integers(tile_n):
    import os
    rng = np.random.default_rng(9)
    for (M, N, K) in RAGGED:
        A, B = int_codes(rng, (M, K)), int_codes(rng, (K, N))
        S, _ = oracle.gemm_rows(A, E4M3, B, E4M3)
        for mode in MODES:
            D, amax = run_fused(A, E4M3, B, E4M3, fp8.FP8_OUT_F32, np.float32(0.5), np.float32(4.0), want_amax=True, mode=mode)
            assert np.array_equal(out_to_f64(D), S / 2.0), (M, N, K, mode)
            assert float(amax) == np.max(np.abs(S / 2.0))
        with knob(fp8.FP8_KNOB_GEMM_KERNEL, 1):
            G, _ = run_fused(A, E4M3, B, E4M3, fp8.FP8_OUT_F32, np.float32(0.5), np.float32(4.0))
        assert np.array_equal(out_to_f64(G), S / 2.0)


@pytest.mark.parametrize("mode", MODES)
def test_any_n_with_b_stored_n_by_k_and_unaligned_outputs(mode, tile_n):
    """With B stored N x K (weights kept [out, in]) the tiled kernel takes any N, e.g. a vocabulary
    size, and an output or a per-column factor vector that does not start on a 16-byte boundary: its
    epilogue then stores element by element.  Every output kind, factors per row and per column, the
    output amax; nothing may be written outside D."""
    rng = np.random.default_rng(77)
    for (M, N, K, transA, off) in [(300, 1001, 256, 0, 0), (64, 17, 128, 0, 0), (257, 1, 128, 0, 0),
                                   (128, 50257 // 16, 384, 1, 0), (200, 272, 256, 0, 3), (513, 255, 128, 0, 1)]:
        A = random_codes(rng, (M, K), E4M3)
        B = random_codes(rng, (K, N), E5M2, 0x6F)
        S, T = oracle.gemm_rows(A, E4M3, B, E5M2)
        sA = rng.uniform(0.5, 4.0, M).astype(np.float32)
        sB = rng.uniform(0.5, 4.0, N).astype(np.float32)
        dA = to_dev(np.ascontiguousarray(A.T) if transA else A)
        dB = to_dev(np.ascontiguousarray(B.T))
        c_ref, b = reference(S, T, sA, sB, mode)
        sBbuf = torch.zeros(N + 8, device="cuda")
        sBbuf[off:off + N] = torch.from_numpy(sB).cuda()
        for out_kind in (fp8.FP8_OUT_F32, fp8.FP8_OUT_BF16, fp8.FP8_OUT_E4M3):
            esz = {fp8.FP8_OUT_F32: 4, fp8.FP8_OUT_BF16: 2, fp8.FP8_OUT_E4M3: 1}[out_kind]
            pad = 4096 // esz
            buf = torch.zeros(2 * pad + M * N + 8, dtype=OUT_T[out_kind], device="cuda")
            buf.fill_(7)
            D = buf[pad + off:pad + off + M * N].view(M, N)
            amax = torch.full((1,), -1.0, device="cuda")
            sD = dev_f32(np.float32(448.0 / np.max(np.abs(c_ref)))) if out_kind == fp8.FP8_OUT_E4M3 else None
            fp8.fp8_gemm_fused(dA, E4M3, transA, dB, E5M2, 1, D, out_kind, dev_f32(sA), sBbuf[off:off + N], sD, amax,
                               flags_of(mode))
            torch.cuda.synchronize()
            what = "any N %s transA %d offset %d out %d %s" % ((M, N, K), transA, off, out_kind, mode)
            plan = fp8.fp8_gemm_plan(dA, transA, dB, 1, D, sBbuf[off:off + N])
            if N % 16 or off:                                   # the matrix-core kernel with element-wise stores
                assert plan & fp8.FP8_PLAN_ELEMENTWISE_STORES and plan & 15 in (fp8.FP8_PLAN_TILED_256x256, fp8.FP8_PLAN_TILED_256x128, fp8.FP8_PLAN_TILED_MIXED), what
            assert bool((buf[:pad + off] == 7).all()) and bool((buf[pad + off + M * N:] == 7).all()), what + ": wrote outside D"
            if out_kind == fp8.FP8_OUT_E4M3:
                check_fp8_bytes(D.cpu().numpy(), c_ref, b, np.float32(sD.item()), E4M3, what,
                                min_exact=0.99 if mode == "f16" else 0.80)
            else:
                check_wide(D, S, T, sA, sB, out_kind, mode, what)
            check_amax(np.float32(amax.item()), c_ref, b, what)


def test_random_shapes_layouts_formats_and_modes_exact_on_integers(tile_n):
    """A seeded sweep over shapes (any M, N a multiple of 16 or not, K a multiple of 128 or not: tiled
    and generic kernel), storage orders, format pairs, modes and output kinds.  Operands are small
    integers, so every sum is exact in fp32 in any order and the output must equal the oracle's."""
    rng = np.random.default_rng(20260)
    for case in range(24):
        M = int(rng.integers(1, 700))
        N = int(rng.integers(1, 45)) * 16 if case % 4 else int(rng.integers(1, 700))
        K = int(rng.integers(1, 9)) * 128 if case % 5 else int(rng.integers(1, 600))
        transA, transB = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        fmtA, fmtB = (E4M3, E5M2)[int(rng.integers(0, 2))], (E4M3, E5M2)[int(rng.integers(0, 2))]
        mode = MODES[case % len(MODES)]
        out_kind = (fp8.FP8_OUT_F32, fp8.FP8_OUT_BF16)[int(rng.integers(0, 2))]
        A = oracle.quantize(rng.integers(-4, 5, (M, K)).astype(np.float32), fmtA, 1.0)
        B = oracle.quantize(rng.integers(-4, 5, (K, N)).astype(np.float32), fmtB, 1.0)
        S, _ = oracle.gemm_rows(A, fmtA, B, fmtB)
        D, amax = run_fused(A, fmtA, B, fmtB, out_kind, np.float32(2.0), np.float32(0.25), want_amax=True, mode=mode,
                            transA=transA, transB=transB)
        what = "case %d: %s layout %d%d formats %d%d %s out %d" % (case, (M, N, K), transA, transB, fmtA, fmtB, mode, out_kind)
        want = S * 2.0                                      # 1 / (2 * 0.25)
        if out_kind == fp8.FP8_OUT_BF16:
            want = torch.from_numpy(want.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
        assert np.array_equal(out_to_f64(D), want), what
        assert float(amax) == np.max(np.abs(S * 2.0)), what


def test_wgrad_of_the_ffn_up_layer_full_size():
    """dW[49152 x 12288] = dY^T X with dY [8192 x 49152] (bf16 -> E5M2) and X [8192 x 12288] (bf16 ->
    E4M3), K = 8192 tokens: the weight-gradient GEMM of the FFN-up layer at full size.  dY is cast
    once, into both storage orders; the product is formed from the plain bytes with transA = 1 and
    from the transposed bytes with transA = 0, with per-tensor factors and with per-row (per output
    channel) factors folded in; sampled outputs against the oracle."""
    X_bits, _ = synth.config4()                       # activations of config 4: 8192 x 12288
    dY_bits, _ = synth.config5()                      # activation gradients of config 5: 8192 x 49152, Laplace
    T_, d_in = X_bits.shape
    d_out = dY_bits.shape[1]
    sX = oracle.scale_from_amax(oracle.amax(X_bits), E4M3)
    sY = oracle.scale_from_amax(oracle.amax(dY_bits), E5M2)
    dX, ddY = to_dev(X_bits), to_dev(dY_bits)
    qX = torch.empty((T_, d_in), dtype=torch.uint8, device="cuda")
    qY = torch.empty((T_, d_out), dtype=torch.uint8, device="cuda")
    qYt = torch.empty((d_out, T_), dtype=torch.uint8, device="cuda")
    fp8.fp8_quantize(dX, E4M3, float(sX), qX)
    fp8.fp8_quantize_transpose(ddY, E5M2, dev_f32(sY), qY, qYt)
    torch.cuda.synchronize()
    del dX, ddY
    Yq = oracle.quantize(dY_bits, E5M2, sY)
    Xq = oracle.quantize(X_bits, E4M3, sX)
    del X_bits, dY_bits
    assert np.array_equal(qX.cpu().numpy(), Xq), "cast of X differs"
    assert np.array_equal(qY.cpu().numpy(), Yq), "cast of dY differs"
    assert torch.equal(qYt, qY.t()), "transposed cast of dY differs from the plain one"
    Ytq = np.ascontiguousarray(Yq.T)                  # op(A) = dY^T as an M x K matrix for the oracle
    del Yq
    M, N, K = d_out, d_in, T_
    rng = np.random.default_rng(6)
    pi, pj = sample_points(rng, M, N, 2000)
    S, T = oracle.gemm_points(Ytq, E5M2, Xq, E4M3, pi, pj)
    ti, tj = torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda()
    dW = torch.empty((M, N), dtype=torch.float32, device="cuda")
    row_factor = (0.5 + rng.random(M)).astype(np.float32)          # an extra factor per output channel
    for mode in MODES:
        c_ref, b = reference(S, T, sY, sX, mode)
        bound = b + 0.5 * oracle.ulp(c_ref, oracle.F32)
        for A_dev, transA in ((qY, 1), (qYt, 0)):
            fp8.fp8_gemm_ex(A_dev, E5M2, transA, qX, E4M3, 0, dW, float(sY), float(sX), flags_of(mode))
            torch.cuda.synchronize()
            err = np.abs(dW[ti, tj].cpu().numpy().astype(np.float64) - c_ref)
            assert np.all(err <= bound), "wgrad %s transA=%d: worst err/bound %.3g" % (mode, transA, np.max(err / bound))
        sA_rows = (float(sY) * row_factor).astype(np.float32)
        fp8.fp8_gemm_fused(qY, E5M2, 1, qX, E4M3, 0, dW, fp8.FP8_OUT_F32, dev_f32(sA_rows), dev_f32(sX), None, None,
                           flags_of(mode))
        torch.cuda.synchronize()
        alpha = 1.0 / (sA_rows[pi].astype(np.float64) * float(sX))
        c_ref2 = alpha * S
        bound2 = REL[mode] * alpha * np.abs(T) + 0.5 * oracle.ulp(c_ref2, oracle.F32)
        err = np.abs(dW[ti, tj].cpu().numpy().astype(np.float64) - c_ref2)
        assert np.all(err <= bound2), "wgrad per-row factors %s: worst err/bound %.3g" % (mode, np.max(err / bound2))


def test_seeded_sweep_over_plans_and_epilogues_exact_on_integers():
    """Shapes, storage orders, format pairs, both modes, every output kind, per-tensor / per-row /
    per-column power-of-two factors and the output maximum, with the dispatcher left alone or pushed
    by the knobs onto each of its kernels (either tile width, both widths in one launch, the
    any-shape kernel).  Operands are small integers: every sum and every quotient is exact, so the
    outputs (FP8 bytes included) and the maximum must equal the oracle's, and nothing may be written
    outside D."""
    rng = np.random.default_rng(20261)
    seen = {}
    for case in range(96):
        kind = case % 4
        if kind == 3:
            M, N, K = int(rng.integers(1, 700)), int(rng.integers(1, 900)), int(rng.integers(1, 500))
        else:
            M = int(rng.integers(1, 7)) * 128 + 16 * int(rng.integers(0, 8)) * (kind == 0)
            N = int(rng.integers(2, 12)) * 128 + 16 * int(rng.integers(0, 8)) * (kind != 1)
            K = int(rng.integers(1, 10)) * 64 + 16 * int(rng.integers(0, 4)) * (kind == 2)
        transA, transB = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        if kind != 3 and transA:
            M = (M + 15) // 16 * 16
        fmtA, fmtB = (E4M3, E5M2)[int(rng.integers(0, 2))], (E4M3, E5M2)[int(rng.integers(0, 2))]
        mode = MODES[int(rng.integers(0, len(MODES)))]
        out_kind = int(rng.integers(0, 4))
        per_row, per_col = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        knobs = {fp8.FP8_KNOB_MIXED: int(rng.integers(0, 3)), fp8.FP8_KNOB_TILE_N: (0, 0, 128, 256)[int(rng.integers(0, 4))],
                 fp8.FP8_KNOB_GEMM_KERNEL: (0, 0, 0, 2)[int(rng.integers(0, 4))]}
        ai = rng.integers(-3, 4, (M, K)).astype(np.float32)
        bi = rng.integers(-3, 4, (K, N)).astype(np.float32)
        A, B = oracle.quantize(ai, fmtA, 1.0), oracle.quantize(bi, fmtB, 1.0)
        S = ai.astype(np.float64) @ bi.astype(np.float64)
        sA = (2.0 ** rng.integers(-2, 3, M if per_row else 1)).astype(np.float32)
        sB = (2.0 ** rng.integers(-2, 3, N if per_col else 1)).astype(np.float32)
        c = S / (sA.astype(np.float64)[:, None] if per_row else float(sA[0])) / (sB.astype(np.float64)[None, :] if per_col else float(sB[0]))
        sD = np.float32(2.0 ** int(rng.integers(-3, 2)))
        if out_kind >= fp8.FP8_OUT_E4M3:
            want = oracle.quantize(c.astype(np.float32), E4M3 if out_kind == fp8.FP8_OUT_E4M3 else E5M2, sD)
        elif out_kind == fp8.FP8_OUT_BF16:
            want = torch.from_numpy(c).to(torch.bfloat16).double().numpy()
        else:
            want = c
        dA = to_dev(np.ascontiguousarray(A.T) if transA else A)
        dB = to_dev(np.ascontiguousarray(B.T) if transB else B)
        guard = 64
        flat = torch.full((M * N + 2 * guard,), 5, dtype=OUT_T[out_kind], device="cuda")
        D = flat[guard:guard + M * N].view(M, N)
        amax = torch.full((1,), -1.0, device="cuda")
        what = "case %d: %s layout %d%d formats %d%d %s out %d per-row %d per-col %d knobs %s" % (
            case, (M, N, K), transA, transB, fmtA, fmtB, mode, out_kind, per_row, per_col, list(knobs.values()))
        old = {k: fp8.fp8_set_knob(k, v) for k, v in knobs.items()}
        try:
            plan = fp8.fp8_gemm_plan(dA, transA, dB, transB, D, dev_f32(sB) if per_col else None) & 15
            seen[plan] = seen.get(plan, 0) + 1
            fp8.fp8_gemm_fused(dA, fmtA, transA, dB, fmtB, transB, D, out_kind, dev_f32(sA), dev_f32(sB),
                               dev_f32(sD) if out_kind >= fp8.FP8_OUT_E4M3 else None, amax, flags_of(mode))
            torch.cuda.synchronize()
        finally:
            for k, v in old.items():
                fp8.fp8_set_knob(k, v)
        got = D.cpu().numpy() if out_kind >= fp8.FP8_OUT_E4M3 else out_to_f64(D)
        assert np.array_equal(got, want), what + ": %d outputs differ" % np.count_nonzero(got != want)
        assert float(amax.item()) == float(np.max(np.abs(c))), what
        assert bool((flat[:guard] == 5).all()) and bool((flat[guard + M * N:] == 5).all()), what + ": wrote outside D"
    for plan in (fp8.FP8_PLAN_TILED_256x256, fp8.FP8_PLAN_TILED_256x128, fp8.FP8_PLAN_TILED_MIXED, fp8.FP8_PLAN_MFMA_ANY):
        assert seen.get(plan, 0) >= 3, "the sweep did not reach plan %d often enough: %s" % (plan, seen)
