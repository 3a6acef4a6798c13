"""GPU parity: the matrix-core kernel for any shape and alignment (the one the dispatcher takes where
the tiled kernel's conditions fail: K not a multiple of 16, operand rows that do not start on 16-byte
boundaries, unaligned pointers) against the CPU oracle, through fp8_gemm_ex / fp8_gemm_fused.

Acceptance as for fp8_gemm: |C - C_ref| <= 2^-20 * sum_k |a b| / (sA sB) + ulp_out(C_ref) / 2, and
equality where the sums are exact.  FP8_KNOB_GEMM_KERNEL = 2 forces the kernel onto problems the
tiled kernel would take, = 1 forces the plain FMA kernel (an independent second implementation).
The kernel has two forms (128 x 128 tiles, several workgroups per compute unit; 256 x 256 tiles,
pipelined by hand, for problems of many tiles); FP8_KNOB_TILE_N = 128 / 256 forces one, and the
tests run under both."""

import numpy as np
import pytest
import torch

import oracle
import paper_2209_05433_amd as fp8
from gpu_util import to_dev, out_to_f64, knob

pytestmark = pytest.mark.gpu

E4M3, E5M2 = fp8.FP8_E4M3, fp8.FP8_E5M2
OUT = {fp8.FP8_F32: torch.float32, fp8.FP8_BF16: torch.bfloat16}
ANY = fp8.FP8_PLAN_MFMA_ANY


@pytest.fixture(params=[128, 256], ids=["tile128", "tile256"])
def form(request):
    with knob(fp8.FP8_KNOB_TILE_N, request.param):
        yield request.param


def random_codes(rng, shape, fmt, top=None):
    top = top if top is not None else (0x7E if fmt == E4M3 else 0x5F)
    return rng.integers(0, top + 1, size=shape).astype(np.uint8) | (rng.integers(0, 2, size=shape).astype(np.uint8) << 7)


def stored(X, trans):
    return np.ascontiguousarray(X.T) if trans else X


def bound_check(C, S, T, sA, sB, out_dtype, what):
    c_ref, bound = oracle.gemm_bound(S, T, sA, sB, out_dtype)
    err = np.abs(out_to_f64(C) - c_ref)
    assert np.all(err <= bound), "%s: worst err/bound %.3g" % (what, np.max(err / bound))


@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_odd_shapes_every_storage_order_exact_on_integers(transA, transB, form):
    """Shapes with nothing aligned (odd M, N, K; one to several tiles; K shorter than a stage, K with
    a ragged last 16-byte piece), small integer operands: every sum is exact, the result must equal
    the oracle's, and nothing may be written outside C."""
    rng = np.random.default_rng(40 + 2 * transA + transB)
    for (M, N, K) in [(1, 1, 1), (5, 3, 7), (129, 127, 33), (131, 257, 95), (300, 401, 777), (64, 1001, 50), (515, 130, 1),
                      (257, 513, 64), (260, 250, 129), (77, 300, 193), (258, 31, 256), (33, 290, 321)]:
        fmtA, fmtB = ((E4M3, E5M2), (E5M2, E4M3))[(M + N) % 2]
        A = oracle.quantize(rng.integers(-4, 5, (M, K)).astype(np.float32), fmtA, 1.0)
        B = oracle.quantize(rng.integers(-4, 5, (K, N)).astype(np.float32), fmtB, 1.0)
        S, _ = oracle.gemm_rows(A, fmtA, B, fmtB)
        dA, dB = to_dev(stored(A, transA)), to_dev(stored(B, transB))
        for out_dtype in (fp8.FP8_F32, fp8.FP8_BF16):
            guard = 64
            flat = torch.full((M * N + 2 * guard,), 77.0, dtype=OUT[out_dtype], device="cuda")
            C = flat[guard:guard + M * N].view(M, N)
            if K % 16 or (not transB and N % 16) or (transA and M % 16):
                assert fp8.fp8_gemm_plan(dA, transA, dB, transB, C) == ANY, (M, N, K)
            with knob(fp8.FP8_KNOB_GEMM_KERNEL, 2):
                fp8.fp8_gemm_ex(dA, fmtA, transA, dB, fmtB, transB, C, 2.0, 0.25)
            torch.cuda.synchronize()
            want = S * 2.0
            if out_dtype == fp8.FP8_BF16:
                want = torch.from_numpy(want.astype(np.float32)).to(torch.bfloat16).double().numpy()
            assert np.array_equal(out_to_f64(C), want), ((M, N, K), transA, transB, out_dtype)
            assert torch.all(flat[:guard] == 77.0) and torch.all(flat[guard + M * N:] == 77.0), "wrote outside C"


@pytest.mark.parametrize("offA,offB", [(1, 0), (0, 3), (5, 9), (15, 15)])
def test_operands_at_any_address(offA, offB, form):
    """Operand pointers that are not 16-byte aligned (views into larger byte buffers), aligned shapes:
    the dispatcher must choose this kernel by itself, and the result must meet the bound."""
    rng = np.random.default_rng(7 + offA + 16 * offB)
    M, N, K = 384, 272, 320
    A, B = random_codes(rng, (M, K), E4M3), random_codes(rng, (K, N), E5M2)
    S, T = oracle.gemm_rows(A, E4M3, B, E5M2)
    bufA = torch.zeros(M * K + 32, dtype=torch.uint8, device="cuda")
    bufB = torch.zeros(K * N + 32, dtype=torch.uint8, device="cuda")
    dA = bufA[offA:offA + M * K].view(M, K)
    dB = bufB[offB:offB + K * N].view(K, N)
    dA.copy_(to_dev(A)); dB.copy_(to_dev(B))
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    assert fp8.fp8_gemm_plan(dA, 0, dB, 0, C) == ANY
    fp8.fp8_gemm_ex(dA, E4M3, 0, dB, E5M2, 0, C, 3.0, 0.5)
    torch.cuda.synchronize()
    bound_check(C, S, T, 3.0, 0.5, fp8.FP8_F32, "offsets %d, %d" % (offA, offB))


@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_random_codes_forced_on_a_tiled_problem_and_against_the_other_kernels(transA, transB, form):
    """A problem the tiled kernel takes (512 x 384 x 640), forced through this kernel: within the
    bound of the oracle, like the tiled kernel and the plain FMA kernel on the same bytes."""
    rng = np.random.default_rng(90 + 2 * transA + transB)
    M, N, K = 512, 384, 640
    A, B = random_codes(rng, (M, K), E4M3), random_codes(rng, (K, N), E4M3)
    S, T = oracle.gemm_rows(A, E4M3, B, E4M3)
    dA, dB = to_dev(stored(A, transA)), to_dev(stored(B, transB))
    for kernel, label in ((2, "any-shape"), (0, "tiled"), (1, "FMA")):
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        with knob(fp8.FP8_KNOB_GEMM_KERNEL, kernel):
            fp8.fp8_gemm_ex(dA, E4M3, transA, dB, E4M3, transB, C, 1.5, 0.75)
        torch.cuda.synchronize()
        bound_check(C, S, T, 1.5, 0.75, fp8.FP8_F32, label)


def test_vocabulary_sized_weight_stored_in_by_out(form):
    """The shape class this kernel exists for: B stored K x N with an odd N (a vocabulary projection
    with the weight kept [in, out]), several hundred tiles, K a multiple of nothing in particular;
    sampled rows against the oracle."""
    rng = np.random.default_rng(5)
    M, N, K = 640, 5027, 1237
    A, B = random_codes(rng, (M, K), E4M3, 0x5F), random_codes(rng, (K, N), E4M3, 0x5F)
    rows = np.sort(rng.choice(M, 24, replace=False))
    S, T = oracle.gemm_rows(A, E4M3, B, E4M3, rows)
    dA, dB = to_dev(A), to_dev(B)
    for out_dtype in (fp8.FP8_BF16, fp8.FP8_F32):
        C = torch.empty((M, N), dtype=OUT[out_dtype], device="cuda")
        assert fp8.fp8_gemm_plan(dA, 0, dB, 0, C) == ANY
        fp8.fp8_gemm_ex(dA, E4M3, 0, dB, E4M3, 0, C, 4.0, 2.0, fp8.FP8_GEMM_MFMA8 if out_dtype == fp8.FP8_F32 else 0)
        torch.cuda.synchronize()
        bound_check(C[torch.from_numpy(rows).cuda()], S, T, 4.0, 2.0, out_dtype, "N = 5027, out %d" % out_dtype)


def test_many_tiles_dispatchers_own_choice_of_form():
    """256 tiles of 256 x 256 with an odd N and K = 520 (eight whole stages and a ragged ninth): the
    dispatcher takes the wide form by itself (no knob set); sampled rows against the oracle, and
    the other form must give the same bits (same products, same order of accumulation)."""
    rng = np.random.default_rng(2024)
    M, N, K = 4096, 4081, 520
    A, B = random_codes(rng, (M, K), E5M2, 0x5F), random_codes(rng, (K, N), E4M3, 0x5F)
    rows = np.sort(rng.choice(M, 16, replace=False))
    S, T = oracle.gemm_rows(A, E5M2, B, E4M3, rows)
    dA, dB = to_dev(A), to_dev(B)
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    assert fp8.fp8_get_knob(fp8.FP8_KNOB_TILE_N) == 0
    assert fp8.fp8_gemm_plan(dA, 0, dB, 0, C) == ANY
    fp8.fp8_gemm_ex(dA, E5M2, 0, dB, E4M3, 0, C, 8.0, 0.5)
    torch.cuda.synchronize()
    bound_check(C[torch.from_numpy(rows).cuda()], S, T, 8.0, 0.5, fp8.FP8_F32, "4096 x 4081 x 520")
    C2 = torch.empty_like(C)
    with knob(fp8.FP8_KNOB_TILE_N, 128):
        fp8.fp8_gemm_ex(dA, E5M2, 0, dB, E4M3, 0, C2, 8.0, 0.5)
    torch.cuda.synchronize()
    assert torch.equal(C, C2)


def test_special_values_and_zero_padding(form):
    """NaN and infinity in the operands propagate as IEEE arithmetic says, also next to the zero
    padding of a ragged K and ragged tile edges: the padding must not turn an infinity into NaN."""
    M, N, K = 70, 45, 50
    A = np.full((M, K), oracle.encode(E5M2, 1.0), dtype=np.uint8)
    B = np.full((K, N), oracle.encode(E4M3, 2.0), dtype=np.uint8)
    A[3, K - 1] = 0x7C                      # +inf (E5M2) in the last, partly padded 16-byte piece of its row
    A[9, 0] = 0x7F                          # NaN (E5M2)
    B[K - 1, 7] = 0x7F                      # NaN (E4M3) in the last K-row
    S, _ = oracle.gemm_rows(A, E5M2, B, E4M3)
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    fp8.fp8_gemm_ex(to_dev(A), E5M2, 0, to_dev(B), E4M3, 0, C, 1.0, 1.0)
    torch.cuda.synchronize()
    got = out_to_f64(C)
    assert np.array_equal(np.isnan(got), np.isnan(S)) and np.array_equal(np.isinf(got), np.isinf(S))
    ok = np.isfinite(S)
    assert np.array_equal(got[ok], S[ok])
    assert np.all(np.isinf(got[3, np.arange(N) != 7])) and np.all(np.isnan(got[9])) and np.all(np.isnan(got[:, 7]))


def test_fused_epilogue_on_a_ragged_problem(form):
    """Per-row and per-column factors, FP8 output with output scale and output amax, on a shape only
    this kernel takes; integers, so the FP8 bytes must be the oracle's."""
    rng = np.random.default_rng(77)
    M, N, K = 200, 150, 90
    A = oracle.quantize(rng.integers(-3, 4, (M, K)).astype(np.float32), E4M3, 1.0)
    B = oracle.quantize(rng.integers(-3, 4, (K, N)).astype(np.float32), E4M3, 1.0)
    S, _ = oracle.gemm_rows(A, E4M3, B, E4M3)
    sA = (2.0 ** rng.integers(-2, 3, M)).astype(np.float32)
    sB = (2.0 ** rng.integers(-2, 3, N)).astype(np.float32)
    c = S / (sA.astype(np.float64)[:, None] * sB.astype(np.float64)[None, :])
    sD = np.float32(0.5)
    want = oracle.quantize(c.astype(np.float32), E4M3, sD)
    D = torch.empty((M, N), dtype=torch.uint8, device="cuda")
    amax = torch.zeros(1, device="cuda")
    fp8.fp8_gemm_fused(to_dev(A), E4M3, 0, to_dev(B), E4M3, 0, D, fp8.FP8_OUT_E4M3, to_dev(sA), to_dev(sB),
                       to_dev(np.array([sD])), amax)
    torch.cuda.synchronize()
    assert np.array_equal(D.cpu().numpy(), want)
    assert float(amax.item()) == float(np.max(np.abs(c)))
