"""GPU parity: fp8_gemm_splitk (K cut into slices, fp32 partial sums in a workspace, added in slice
order) against the CPU oracle, to the bound of fp8_gemm_ex:
    |C - C_ref| <= 2^-20 * sum_k |a_ik b_kj| / (sA sB) + ulp_out(C_ref) / 2
(2^-10 with the FP8 matrix-core instructions); exact where the sums are exact; the same bits in
every run."""
import numpy as np
import pytest
import torch

import oracle
import paper_2209_05433_amd as fp8
from gpu_util import to_dev, out_to_f64, knob, freivalds_blocks

pytestmark = pytest.mark.gpu

E4M3, E5M2 = fp8.FP8_E4M3, fp8.FP8_E5M2
OUT = {fp8.FP8_F32: torch.float32, fp8.FP8_BF16: torch.bfloat16}
REL = {0: 2.0 ** -20, fp8.FP8_GEMM_MFMA8: 2.0 ** -10}


def random_codes(rng, shape, fmt, top=None):
    top = top if top is not None else (0x7E if fmt == E4M3 else 0x5F)
    return rng.integers(0, top + 1, size=shape).astype(np.uint8) | (rng.integers(0, 2, size=shape).astype(np.uint8) << 7)


def splitk(dA, fmtA, tA, dB, fmtB, tB, M, N, K, out_dtype, sA, sB, flags, splits, fill=None, slack=0):
    need = fp8.fp8_gemm_splitk_workspace_size(M, N, K, tA, tB, splits)
    ws = torch.full((need + slack,), 0xFF, dtype=torch.uint8, device="cuda") if need + slack else None   # NaN patterns: stale reads would show
    C = torch.empty((M, N), dtype=OUT[out_dtype], device="cuda")
    if fill is not None:
        C.fill_(fill)
    fp8.fp8_gemm_splitk(dA, fmtA, tA, dB, fmtB, tB, C, sA, sB, ws, flags, splits)
    torch.cuda.synchronize()
    return C, need


@pytest.mark.parametrize("flags", [0, fp8.FP8_GEMM_MFMA8])
@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_integer_operands_are_exact_for_every_slice_count(transA, transB, flags):
    """Integers in [-4, 4]: every partial sum is exact in fp32 whatever the slicing, so every slice
    count, including those that leave a short last slice and a K that ends inside a stage pair, must
    reproduce the oracle exactly."""
    rng = np.random.default_rng(11 + 2 * transA + transB)
    for (M, N, K) in [(256, 384, 128 * 20), (300, 200, 64 * 37), (512, 256, 2000)]:
        ai = rng.integers(-4, 5, (M, K)).astype(np.float32)
        bi = rng.integers(-4, 5, (K, N)).astype(np.float32)
        Aq, Bq = oracle.quantize(ai, E4M3, 1.0), oracle.quantize(bi, E4M3, 1.0)
        S, _ = oracle.gemm_rows(Aq, E4M3, Bq, E4M3)
        dA = to_dev(np.ascontiguousarray(Aq.T) if transA else Aq)
        dB = to_dev(np.ascontiguousarray(Bq.T) if transB else Bq)
        for splits in (0, 1, 2, 3, 5, 7, 16, 64):
            C, need = splitk(dA, E4M3, transA, dB, E4M3, transB, M, N, K, fp8.FP8_F32, 2.0, 0.25, flags, splits, fill=9.0)
            assert np.array_equal(out_to_f64(C), S * 2.0), (M, N, K, splits)
            assert need % (4 * M * N) == 0 and need // (4 * M * N) <= max(1, 64 if splits == 0 else splits)


@pytest.mark.parametrize("flags", [0, fp8.FP8_GEMM_MFMA8])
@pytest.mark.parametrize("out_dtype", [fp8.FP8_F32, fp8.FP8_BF16])
def test_random_codes_within_the_bound_and_bit_identical_run_to_run(out_dtype, flags):
    rng = np.random.default_rng(5)
    M, N, K = 384, 520, 128 * 24           # B stored N x K, N not a multiple of 16
    A, B = random_codes(rng, (M, K), E5M2), random_codes(rng, (K, N), E4M3)
    S, T = oracle.gemm_rows(A, E5M2, B, E4M3)
    sA, sB = np.float32(3.1), np.float32(0.07)
    dA, dBt = to_dev(A), to_dev(np.ascontiguousarray(B.T))
    for splits in (0, 4, 9):
        for dev_scales in (False, True):
            a = torch.tensor([sA], device="cuda") if dev_scales else float(sA)
            b = torch.tensor([sB], device="cuda") if dev_scales else float(sB)
            C1, _ = splitk(dA, E5M2, 0, dBt, E4M3, 1, M, N, K, out_dtype, a, b, flags, splits)
            C2, _ = splitk(dA, E5M2, 0, dBt, E4M3, 1, M, N, K, out_dtype, a, b, flags, splits)
            assert torch.equal(C1, C2), "two runs differ"
            c_ref, alpha = oracle.unscale(S, sA, sB)
            bound = REL[flags] * alpha * T + 0.5 * oracle.ulp(c_ref, out_dtype)
            err = np.abs(out_to_f64(C1) - c_ref)
            assert np.all(err <= bound), "splits=%d: worst err/bound %.3g" % (splits, np.max(err / bound))


def test_ragged_n_and_unaligned_workspace_take_the_elementwise_path():
    """N not a multiple of 4 (rows of the slices do not start on 16-byte boundaries) and a workspace
    that is only 4-byte aligned."""
    rng = np.random.default_rng(21)
    M, N, K = 256, 203, 128 * 8
    ai = rng.integers(-4, 5, (M, K)).astype(np.float32)
    bi = rng.integers(-4, 5, (K, N)).astype(np.float32)
    Aq, Bq = oracle.quantize(ai, E4M3, 1.0), oracle.quantize(bi, E4M3, 1.0)
    S, _ = oracle.gemm_rows(Aq, E4M3, Bq, E4M3)
    dA, dBt = to_dev(Aq), to_dev(np.ascontiguousarray(Bq.T))
    for out_dtype in (fp8.FP8_F32, fp8.FP8_BF16):
        need = fp8.fp8_gemm_splitk_workspace_size(M, N, K, 0, 1, 4)
        assert need == 4 * M * N * 4
        buf = torch.full((need + 16,), 0xFF, dtype=torch.uint8, device="cuda")
        C = torch.zeros((M, N), dtype=OUT[out_dtype], device="cuda")
        fp8.fp8_gemm_splitk(dA, E4M3, 0, dBt, E4M3, 1, C, 1.0, 1.0, buf[4:], 0, 4)
        torch.cuda.synchronize()
        want = torch.from_numpy(S).to(OUT[out_dtype]).double().numpy()      # integers below 2^24; bf16 rounds
        assert np.array_equal(out_to_f64(C), want)


def test_problems_outside_the_tiled_kernel_need_no_workspace():
    rng = np.random.default_rng(2)
    M, N, K = 70, 33, 100                               # K % 16 != 0: plain FMA kernel
    A, B = random_codes(rng, (M, K), E4M3), random_codes(rng, (K, N), E4M3)
    S, T = oracle.gemm_rows(A, E4M3, B, E4M3)
    assert fp8.fp8_gemm_splitk_workspace_size(M, N, K, 0, 0, 8) == 0
    C, _ = splitk(to_dev(A), E4M3, 0, to_dev(B), E4M3, 0, M, N, K, fp8.FP8_F32, 1.0, 1.0, 0, 8)
    c_ref, alpha = oracle.unscale(S, 1.0, 1.0)
    assert np.all(np.abs(out_to_f64(C) - c_ref) <= 2.0 ** -20 * T + 0.5 * oracle.ulp(c_ref, oracle.F32))


def test_too_small_a_workspace_is_rejected_before_anything_is_launched():
    M, N, K = 256, 256, 4096
    A = torch.zeros((M, K), dtype=torch.uint8, device="cuda")
    B = torch.zeros((K, N), dtype=torch.uint8, device="cuda")
    C = torch.full((M, N), 3.0, device="cuda")
    need = fp8.fp8_gemm_splitk_workspace_size(M, N, K, 0, 0, 8)
    assert need == 8 * M * N * 4
    with pytest.raises(fp8.Fp8Error) as e:
        fp8.fp8_gemm_splitk(A, E4M3, 0, B, E4M3, 0, C, 1.0, 1.0, torch.empty(need - 4, dtype=torch.uint8, device="cuda"), 0, 8)
    assert e.value.status == fp8.FP8_ERR_INVALID_ARG and str(need) in str(e.value)
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_gemm_splitk(A, E4M3, 0, B, E4M3, 0, C, 1.0, 1.0, None, 0, 8)
    torch.cuda.synchronize()
    assert bool((C == 3.0).all())


def test_weight_gradient_regime_full_size():
    """dW[1024 x 1024] = dY^T X over K = 65536 tokens (E5M2^T x E4M3 -> fp32): 16 tiles, which the
    slices spread over the chip.  Whole rows element by element, every output through block sums,
    identical bits in two runs, and the plain one-workgroup-per-tile call within the same bound."""
    M = N = 1024
    K = 65536
    rng = np.random.default_rng(77)
    dY = random_codes(rng, (K, M), E5M2, 0x4F)          # stored [tokens x out]: A is given as K x M
    X = random_codes(rng, (K, N), E4M3, 0x6F)
    sA, sB = np.float32(1.7e3), np.float32(11.0)
    ddY, dX = to_dev(dY), to_dev(X)
    for flags in (0, fp8.FP8_GEMM_MFMA8):
        C1, need = splitk(ddY, E5M2, 1, dX, E4M3, 0, M, N, K, fp8.FP8_F32, float(sA), float(sB), flags, 0)
        C2, _ = splitk(ddY, E5M2, 1, dX, E4M3, 0, M, N, K, fp8.FP8_F32, float(sA), float(sB), flags, 0)
        assert need >= 8 * M * N * 4, "the automatic choice should cut this problem into many slices"
        assert torch.equal(C1, C2)
        At = np.ascontiguousarray(dY.T)
        rows = np.array([0, 255, 256, 511, 777, 1023])
        S, T = oracle.gemm_rows(At, E5M2, X, E4M3, rows)
        c_ref, alpha = oracle.unscale(S, sA, sB)
        bound = REL[flags] * alpha * T + 0.5 * oracle.ulp(c_ref, oracle.F32)
        err = np.abs(out_to_f64(C1[torch.from_numpy(rows).cuda()]) - c_ref)
        assert np.all(err <= bound), "worst err/bound %.3g" % np.max(err / bound)
        w = freivalds_blocks(C1, At, E5M2, X, E4M3, sA, sB, oracle.F32, rel=REL[flags], label="split-K wgrad")
        print("split-K 1024 x 1024 x 65536 flags=%d: rows worst %.3f, block sums worst %.3f" % (flags, np.max(err / bound), w), flush=True)
        C0 = torch.empty_like(C1)
        fp8.fp8_gemm_ex(ddY, E5M2, 1, dX, E4M3, 0, C0, float(sA), float(sB), flags)
        torch.cuda.synchronize()
        err0 = np.abs(out_to_f64(C0[torch.from_numpy(rows).cuda()]) - c_ref)
        assert np.all(err0 <= bound)
