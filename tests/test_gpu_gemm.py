"""GPU parity: fp8_gemm / fp8_gemm_dscale against the CPU oracle.

Acceptance per output (written into check()):
    |C_gpu - C_ref| <= 2^-20 * sum_k |a_ik b_kj| / (sA sB) + ulp_out(C_ref) / 2
with C_ref the fp64 product of the decoded operands.  Cases whose sums are exact in fp32
must match exactly.  fp8_gemm_mfma8 (FP8 matrix-core instructions, whose adders keep 13 bits
below the largest of each 8 products) is held to its documented bound, 2^-10 in place of
2^-20, and to the exact cases."""

import numpy as np
import pytest
import torch

import oracle
import paper_2209_05433_amd as fp8
from workloads import synth
from gpu_util import to_dev, out_to_f64, knob, freivalds_blocks

pytestmark = pytest.mark.gpu

E4M3, E5M2 = fp8.FP8_E4M3, fp8.FP8_E5M2
OUT = {fp8.FP8_F32: torch.float32, fp8.FP8_BF16: torch.bfloat16}
MIXES = [(E4M3, E4M3), (E5M2, E4M3), (E4M3, E5M2), (E5M2, E5M2)]


MODES = ["f16", "mfma8"]
GEMM = {("f16", False): fp8.fp8_gemm, ("f16", True): fp8.fp8_gemm_dscale,
        ("mfma8", False): fp8.fp8_gemm_mfma8, ("mfma8", True): fp8.fp8_gemm_mfma8_dscale}
REL = {"f16": 2.0 ** -20, "mfma8": 2.0 ** -10}
TILED = (fp8.FP8_PLAN_TILED_256x256, fp8.FP8_PLAN_TILED_256x128, fp8.FP8_PLAN_TILED_MIXED)


def run_gemm(Aq, fmtA, sA, Bq, fmtB, sB, out_dtype, dscale=False, fill=None, mode="f16"):
    A, B = to_dev(Aq), to_dev(Bq)
    C = torch.empty((Aq.shape[0], Bq.shape[1]), dtype=OUT[out_dtype], device="cuda")
    if fill is not None:
        C.fill_(fill)
    if dscale:
        GEMM[mode, True](A, fmtA, torch.tensor([sA], dtype=torch.float32, device="cuda"),
                         B, fmtB, torch.tensor([sB], dtype=torch.float32, device="cuda"), C)
    else:
        GEMM[mode, False](A, fmtA, sA, B, fmtB, sB, C)
    torch.cuda.synchronize()
    return C


def check(C_vals, S, T, sA, sB, out_dtype, what="", mode="f16"):
    c_ref, bound = oracle.gemm_bound(S, T, sA, sB, out_dtype)
    if mode != "f16":      # same form, larger constant: bound = rel * alpha * T + ulp / 2
        bound = bound + (REL[mode] - 2.0 ** -20) * np.abs(T) / (float(np.float32(sA)) * float(np.float32(sB)))
    err = np.abs(C_vals - c_ref)
    ratio = err / bound
    worst = np.nanargmax(ratio) if ratio.size else 0
    assert np.all(err <= bound), "%s: worst err/bound %.3g at flat index %d (got %r want %r)" % (
        what, ratio.flat[worst], worst, C_vals.flat[worst], c_ref.flat[worst])
    return float(ratio.max()) if ratio.size else 0.0


def random_codes(rng, shape, fmt, max_code=None):
    """Uniformly random finite FP8 codes of both signs."""
    top = max_code if max_code is not None else (0x7E if fmt == E4M3 else 0x7B)
    mag = rng.integers(0, top + 1, size=shape).astype(np.uint8)
    return mag | (rng.integers(0, 2, size=shape).astype(np.uint8) << 7)


def quantize_pair(A, B, fmtA, fmtB):
    sA = oracle.scale_from_amax(oracle.amax(A), fmtA)
    sB = oracle.scale_from_amax(oracle.amax(B), fmtB)
    return oracle.quantize(A, fmtA, sA), sA, oracle.quantize(B, fmtB, sB), sB


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", [(256, 256, 512), (512, 256, 128), (256, 768, 1024), (33, 20, 77)])
def test_small_integer_operands_are_exact(shape, mode):
    """Integers in [-4, 4]: every partial sum is an integer below 2^24, alpha is a power of two,
    so fp32 accumulation is exact in any order and the result must equal the oracle's exactly."""
    M, N, K = shape
    rng = np.random.default_rng(M + N + K)
    ai = rng.integers(-4, 5, (M, K)).astype(np.float32)
    bi = rng.integers(-4, 5, (K, N)).astype(np.float32)
    Aq, Bq = oracle.quantize(ai, E4M3, 1.0), oracle.quantize(bi, E4M3, 1.0)
    S, _ = oracle.gemm_rows(Aq, E4M3, Bq, E4M3)
    C = run_gemm(Aq, E4M3, 2.0, Bq, E4M3, 0.25, fp8.FP8_F32, mode=mode)
    assert np.array_equal(out_to_f64(C), S * 2.0)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("fmt", [E4M3, E5M2])
def test_identity_operand_reproduces_decode(fmt, mode):
    """A x I = decode(A) and I x B = decode(B): pins row/column/K placement of every lane."""
    rng = np.random.default_rng(3)
    n = 256
    eye = np.zeros((n, n), dtype=np.uint8)
    eye[np.arange(n), np.arange(n)] = oracle.encode(E4M3, 1.0)
    X = random_codes(rng, (n, n), fmt)
    vals = oracle.decode_all(fmt)[X]
    C = run_gemm(X, fmt, 1.0, eye, E4M3, 1.0, fp8.FP8_F32, mode=mode)
    assert np.array_equal(out_to_f64(C), vals)
    C = run_gemm(eye, E4M3, 1.0, X, fmt, 1.0, fp8.FP8_F32, mode=mode)
    assert np.array_equal(out_to_f64(C), vals)


@pytest.mark.parametrize("mode", MODES)
def test_one_hot_probes_over_a_multi_tile_problem(mode):
    """Single non-zero product placed at seeded positions of a 512 x 768 x 384 problem."""
    M, N, K = 512, 768, 384
    rng = np.random.default_rng(12)
    for _ in range(6):
        i, j, k = int(rng.integers(M)), int(rng.integers(N)), int(rng.integers(K))
        A = np.zeros((M, K), dtype=np.uint8)
        B = np.zeros((K, N), dtype=np.uint8)
        A[i, k] = oracle.encode(E4M3, 3.0)
        B[k, j] = oracle.encode(E4M3, -5.0)
        B[(k + 1) % K, j] = oracle.encode(E4M3, 7.0)        # must not contribute
        C = out_to_f64(run_gemm(A, E4M3, 1.0, B, E4M3, 1.0, fp8.FP8_F32, fill=123.0, mode=mode))
        want = np.zeros((M, N))
        want[i, j] = -15.0
        assert np.array_equal(C, want), (i, j, k)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("out_dtype", [fp8.FP8_F32, fp8.FP8_BF16])
@pytest.mark.parametrize("fmtA,fmtB", MIXES)
def test_random_codes_all_format_mixes(fmtA, fmtB, out_dtype, mode):
    """Random finite codes (whole dynamic range of E4M3; E5M2 limited so that sums stay finite)."""
    rng = np.random.default_rng(100 + 10 * fmtA + fmtB)
    M, N, K = 256, 512, 640
    A = random_codes(rng, (M, K), fmtA, 0x7E if fmtA == E4M3 else 0x5F)
    B = random_codes(rng, (K, N), fmtB, 0x7E if fmtB == E4M3 else 0x5F)
    S, T = oracle.gemm_rows(A, fmtA, B, fmtB)
    sA, sB = np.float32(3.7), np.float32(0.011)
    for dscale in (False, True):
        C = run_gemm(A, fmtA, sA, B, fmtB, sB, out_dtype, dscale=dscale, mode=mode)
        check(out_to_f64(C), S, T, sA, sB, out_dtype, "mix %d x %d" % (fmtA, fmtB), mode=mode)


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 2), (37, 53, 300), (257, 255, 129), (64, 64, 4096), (300, 17, 64)])
def test_ragged_shapes_generic_kernel(shape):
    M, N, K = shape
    rng = np.random.default_rng(M * 7 + N)
    A = random_codes(rng, (M, K), E5M2, 0x5F)
    B = random_codes(rng, (K, N), E4M3)
    S, T = oracle.gemm_rows(A, E5M2, B, E4M3)
    for out_dtype in (fp8.FP8_F32, fp8.FP8_BF16):
        C = run_gemm(A, E5M2, 0.5, B, E4M3, 8.0, out_dtype)
        check(out_to_f64(C), S, T, 0.5, 8.0, out_dtype, str(shape))


def test_generic_and_fast_kernels_agree_within_bound():
    rng = np.random.default_rng(31)
    M, N, K = 256, 256, 256
    A, B = random_codes(rng, (M, K), E4M3), random_codes(rng, (K, N), E4M3)
    S, T = oracle.gemm_rows(A, E4M3, B, E4M3)
    with knob(fp8.FP8_KNOB_GEMM_KERNEL, 1):
        Cg = run_gemm(A, E4M3, 1.0, B, E4M3, 1.0, fp8.FP8_F32)
    Cf = run_gemm(A, E4M3, 1.0, B, E4M3, 1.0, fp8.FP8_F32)
    C8 = run_gemm(A, E4M3, 1.0, B, E4M3, 1.0, fp8.FP8_F32, mode="mfma8")
    check(out_to_f64(Cg), S, T, 1.0, 1.0, fp8.FP8_F32, "generic")
    check(out_to_f64(Cf), S, T, 1.0, 1.0, fp8.FP8_F32, "tiled, fp16 instructions")
    check(out_to_f64(C8), S, T, 1.0, 1.0, fp8.FP8_F32, "tiled, FP8 instructions", mode="mfma8")


def test_empty_and_zero_k():
    A = np.zeros((256, 0), dtype=np.uint8)
    B = np.zeros((0, 256), dtype=np.uint8)
    C = run_gemm(A, E4M3, 1.0, B, E4M3, 1.0, fp8.FP8_BF16, fill=5.0)
    assert torch.count_nonzero(C).item() == 0
    C = run_gemm(np.zeros((0, 8), dtype=np.uint8), E4M3, 1.0, np.zeros((8, 4), dtype=np.uint8), E4M3, 1.0, fp8.FP8_F32)
    assert C.numel() == 0
    # the one-call form on the same degenerate shapes: K = 0 gives amax 0, scale 1 and a zero product
    amax, scale = torch.full((2,), -1.0, device="cuda"), torch.zeros(2, device="cuda")
    ws = torch.zeros(2 * fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
    a, b = torch.empty((16, 0), dtype=torch.bfloat16, device="cuda"), torch.empty((0, 32), dtype=torch.bfloat16, device="cuda")
    C = torch.full((16, 32), 5.0, dtype=torch.float32, device="cuda")
    fp8.fp8_scaled_gemm(a, E4M3, False, b, E5M2, False, torch.empty((16, 0), dtype=torch.uint8, device="cuda"),
                        torch.empty((0, 32), dtype=torch.uint8, device="cuda"), amax, scale, ws, C)
    torch.cuda.synchronize()
    assert torch.count_nonzero(C).item() == 0 and amax.tolist() == [0.0, 0.0] and scale.tolist() == [1.0, 1.0]
    a = torch.ones((0, 8), dtype=torch.float32, device="cuda"); b = torch.full((8, 4), -3.0, dtype=torch.float32, device="cuda")
    qb = torch.empty((8, 4), dtype=torch.uint8, device="cuda")
    fp8.fp8_scaled_gemm(a, E4M3, False, b, E4M3, False, torch.empty((0, 8), dtype=torch.uint8, device="cuda"), qb, amax, scale, ws,
                        torch.empty((0, 4), dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    assert amax.tolist() == [0.0, 3.0] and bool((qb == 0xFE).all())          # -3 * (448 / 3) = -448


@pytest.mark.parametrize("mode", MODES)
def test_non_finite_operands_keep_their_class(mode):
    rng = np.random.default_rng(2)
    M, N, K = 256, 256, 128
    A = random_codes(rng, (M, K), E5M2, 0x40)
    B = random_codes(rng, (K, N), E4M3, 0x40)
    A[3, 7] = 0x7C       # +inf (E5M2)
    A[200, 100] = 0x7E   # NaN (E5M2)
    B[5, 9] = 0x7F       # NaN (E4M3)
    S, _ = oracle.gemm_rows(A, E5M2, B, E4M3)
    C = out_to_f64(run_gemm(A, E5M2, 1.0, B, E4M3, 1.0, fp8.FP8_F32, mode=mode))
    assert np.array_equal(np.isnan(C), np.isnan(S))
    assert np.array_equal(np.isposinf(C), np.isposinf(S)) and np.array_equal(np.isneginf(C), np.isneginf(S))


@pytest.mark.parametrize("mode", MODES)
def test_run_to_run_determinism(mode):
    rng = np.random.default_rng(8)
    A, B = random_codes(rng, (512, 1024), E4M3), random_codes(rng, (1024, 512), E4M3)
    C1 = run_gemm(A, E4M3, 1.0, B, E4M3, 1.0, fp8.FP8_F32, mode=mode)
    C2 = run_gemm(A, E4M3, 1.0, B, E4M3, 1.0, fp8.FP8_F32, mode=mode)
    assert torch.equal(C1, C2)


# ---- the five benchmark workloads -------------------------------------------------------------

def test_config1_whole_path_full_check():
    """fp32 N(0,1) 256^3: amax, scale, cast and GEMM on the GPU; every output checked."""
    A, B = synth.config1()
    dA, dB = to_dev(A), to_dev(B)
    amax = torch.zeros(2, device="cuda")
    scale = torch.zeros(2, device="cuda")
    qA = torch.empty(A.shape, dtype=torch.uint8, device="cuda")
    qB = torch.empty(B.shape, dtype=torch.uint8, device="cuda")
    C = torch.empty((256, 256), dtype=torch.float32, device="cuda")
    for t, q, i in ((dA, qA, 0), (dB, qB, 1)):
        fp8.fp8_amax(t, amax[i:i + 1])
        fp8.fp8_scale_from_amax(amax[i:i + 1], E4M3, scale[i:i + 1])
        fp8.fp8_quantize_dscale(t, E4M3, scale[i:i + 1], q)
    fp8.fp8_gemm_dscale(qA, E4M3, scale[0:1], qB, E4M3, scale[1:2], C)
    torch.cuda.synchronize()
    Aq, sA, Bq, sB = quantize_pair(A, B, E4M3, E4M3)
    assert np.array_equal(qA.cpu().numpy(), Aq) and np.array_equal(qB.cpu().numpy(), Bq)
    assert np.float32(scale[0].item()) == sA and np.float32(scale[1].item()) == sB
    S, T = oracle.gemm_rows(Aq, E4M3, Bq, E4M3)
    check(out_to_f64(C), S, T, sA, sB, fp8.FP8_F32, "config 1")


def test_config1_whole_path_in_one_call():
    """fp8_scaled_gemm on config 1 (fp32 inputs) against the oracle's whole path, and on a bf16
    problem with the operands in the other storage orders against the separate calls, bit for bit."""
    A, B = synth.config1()
    dA, dB = to_dev(A), to_dev(B)
    amax, scale = torch.zeros(2, device="cuda"), torch.zeros(2, device="cuda")
    ws = torch.zeros(2 * fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
    qA = torch.empty(A.shape, dtype=torch.uint8, device="cuda")
    qB = torch.empty(B.shape, dtype=torch.uint8, device="cuda")
    C = torch.empty((256, 256), dtype=torch.float32, device="cuda")
    for _ in range(2):                               # the second call finds the workspace as the first left it
        fp8.fp8_scaled_gemm(dA, E4M3, False, dB, E4M3, False, qA, qB, amax, scale, ws, C)
    torch.cuda.synchronize()
    Aq, sA, Bq, sB = quantize_pair(A, B, E4M3, E4M3)
    assert np.array_equal(qA.cpu().numpy(), Aq) and np.array_equal(qB.cpu().numpy(), Bq)
    assert np.float32(scale[0].item()) == sA and np.float32(scale[1].item()) == sB
    assert float(amax[0].item()) == float(np.max(np.abs(A))) and float(amax[1].item()) == float(np.max(np.abs(B)))
    S, T = oracle.gemm_rows(Aq, E4M3, Bq, E4M3)
    check(out_to_f64(C), S, T, sA, sB, fp8.FP8_F32, "config 1, one call")

    g = torch.Generator(device="cuda").manual_seed(9)
    M, N, K = 384, 640, 512
    a = torch.randn((K, M), device="cuda", generator=g).to(torch.bfloat16)          # stored K x M
    b = (torch.randn((N, K), device="cuda", generator=g) * 0.02).to(torch.bfloat16)  # stored N x K
    qa, qb = torch.empty((K, M), dtype=torch.uint8, device="cuda"), torch.empty((N, K), dtype=torch.uint8, device="cuda")
    c1 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    fp8.fp8_scaled_gemm(a, E5M2, True, b, E4M3, True, qa, qb, amax, scale, ws, c1, fp8.FP8_GEMM_MFMA8)
    amax2, scale2 = torch.zeros(2, device="cuda"), torch.zeros(2, device="cuda")
    ws2 = torch.zeros_like(ws)
    qa2, qb2, c2 = torch.empty_like(qa), torch.empty_like(qb), torch.empty_like(c1)
    fp8.fp8_amax_scale_multi((a, b), (E5M2, E4M3), amax2, scale2, ws2)
    fp8.fp8_quantize_multi((a, b), (E5M2, E4M3), scale2, (qa2, qb2))
    fp8.fp8_gemm_ex(qa2, E5M2, True, qb2, E4M3, True, c2, scale2[0:1], scale2[1:2], fp8.FP8_GEMM_MFMA8)
    torch.cuda.synchronize()
    assert torch.equal(amax, amax2) and torch.equal(scale, scale2)
    assert torch.equal(qa, qa2) and torch.equal(qb, qb2) and torch.equal(c1.view(torch.int16), c2.view(torch.int16))
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_scaled_gemm(a, E5M2, True, b, 7, True, qa, qb, amax, scale, ws, c1)


def sample_points(rng, M, N, npts, tile=256):
    """Corners of the matrix, one point in every 256 x 256 tile (up to a cap), random extras."""
    pts = {(0, 0), (0, N - 1), (M - 1, 0), (M - 1, N - 1)}
    tiles = [(i, j) for i in range(0, M, tile) for j in range(0, N, tile)]
    if len(tiles) > npts // 2:
        tiles = [tiles[t] for t in rng.choice(len(tiles), npts // 2, replace=False)]
    for (i0, j0) in tiles:
        pts.add((i0 + int(rng.integers(min(tile, M - i0))), j0 + int(rng.integers(min(tile, N - j0)))))
    while len(pts) < npts:
        pts.add((int(rng.integers(M)), int(rng.integers(N))))
    p = np.array(sorted(pts), dtype=np.int64)
    return p[:, 0], p[:, 1]


def run_config(A_bits, B_bits, fmtA, fmtB, out_dtype, npts, nrows, label, full=False):
    """Whole path on the GPU at the given size; quantised bytes compared exactly, GEMM outputs
    checked at sampled points and whole rows against the oracle, then all of them (`full`: element
    by element; else by block sums)."""
    M, K = A_bits.shape
    N = B_bits.shape[1]
    dA, dB = to_dev(A_bits), to_dev(B_bits)
    amax = torch.zeros(2, device="cuda")
    scale = torch.zeros(2, device="cuda")
    qA = torch.empty((M, K), dtype=torch.uint8, device="cuda")
    qB = torch.empty((K, N), dtype=torch.uint8, device="cuda")
    C = torch.empty((M, N), dtype=OUT[out_dtype], device="cuda")
    for t, q, i, f in ((dA, qA, 0, fmtA), (dB, qB, 1, fmtB)):
        fp8.fp8_amax(t, amax[i:i + 1])
        fp8.fp8_scale_from_amax(amax[i:i + 1], f, scale[i:i + 1])
        fp8.fp8_quantize_dscale(t, f, scale[i:i + 1], q)
    fp8.fp8_gemm_dscale(qA, fmtA, scale[0:1], qB, fmtB, scale[1:2], C)
    torch.cuda.synchronize()
    assert fp8.fp8_gemm_plan(qA, 0, qB, 0, C) & ~fp8.FP8_PLAN_PERSISTENT in TILED, label
    del dA, dB
    Aq, sA, Bq, sB = quantize_pair(A_bits, B_bits, fmtA, fmtB)
    assert np.float32(scale[0].item()) == sA and np.float32(scale[1].item()) == sB, label
    gA, gB = qA.cpu().numpy(), qB.cpu().numpy()
    assert np.array_equal(gA, Aq), label + ": quantised A differs"
    assert np.array_equal(gB, Bq), label + ": quantised B differs"
    rng = np.random.default_rng(M + N + K)
    pi, pj = sample_points(rng, M, N, npts)
    S, T = oracle.gemm_points(Aq, fmtA, Bq, fmtB, pi, pj)
    Cs = out_to_f64(C[torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda()])
    worst = check(Cs, S, T, sA, sB, out_dtype, label + " points")
    C8 = torch.empty_like(C)
    fp8.fp8_gemm_mfma8_dscale(qA, fmtA, scale[0:1], qB, fmtB, scale[1:2], C8)
    torch.cuda.synchronize()
    C8s = out_to_f64(C8[torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda()])
    worst8 = check(C8s, S, T, sA, sB, out_dtype, label + " points (FP8 instructions)", mode="mfma8")
    c_ref, _ = oracle.gemm_bound(S, T, sA, sB, out_dtype)
    alphaT = np.abs(T) / (float(sA) * float(sB))
    print("%s: FP8-instruction path err / (alpha T): max 2^%.1f mean 2^%.1f" % (
        label, np.log2(np.max(np.abs(C8s - c_ref) / alphaT) + 1e-300),
        np.log2(np.mean(np.abs(C8s - c_ref) / alphaT) + 1e-300)), flush=True)
    del C8
    rows = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, nrows)]))[:nrows + 2]
    Sr, Tr = oracle.gemm_rows(Aq, fmtA, Bq, fmtB, rows)
    worst = max(worst, check(out_to_f64(C[torch.from_numpy(rows).cuda()]), Sr, Tr, sA, sB, out_dtype, label + " rows"))
    # every output: element by element where the reference finishes in seconds, else through
    # signed sums over blocks of 256 columns (two seeded sign vectors)
    if full:
        Sf, Tf = oracle.gemm_rows(Aq, fmtA, Bq, fmtB)
        worst = max(worst, check(out_to_f64(C), Sf, Tf, sA, sB, out_dtype, label + " every output"))
    else:
        w = freivalds_blocks(C, Aq, fmtA, Bq, fmtB, sA, sB, out_dtype, label=label)
        print("%s: block sums of every output, two sign vectors: worst err/bound %.3f" % (label, w), flush=True)
    print("%s: worst err/bound %.3f" % (label, worst), flush=True)


def test_config3_small_gpt_forward():
    A, B = synth.config3()
    run_config(A, B, E4M3, E4M3, fp8.FP8_BF16, npts=3000, nrows=6, label="config 3", full=True)


def test_config4_ffn_up_full_size():
    A, B = synth.config4()
    run_config(A, B, E4M3, E4M3, fp8.FP8_BF16, npts=12400, nrows=2, label="config 4")      # a point in each of the 6144 tiles


def test_config5_dgrad_full_size():
    A, B = synth.config5()
    run_config(A, B, E5M2, E4M3, fp8.FP8_F32, npts=3200, nrows=2, label="config 5")        # a point in each of the 1536 tiles


@pytest.mark.parametrize("fmt", [E4M3, E5M2])
def test_config2_quantize_only_full_size(fmt):
    """2^28 bf16 elements with outliers: amax, scale and every output byte compared."""
    h = synth.config2()
    x = to_dev(h)
    amax = torch.zeros(1, device="cuda")
    scale = torch.zeros(1, device="cuda")
    q = torch.empty(h.size, dtype=torch.uint8, device="cuda")
    fp8.fp8_amax(x, amax)
    fp8.fp8_scale_from_amax(amax, fmt, scale)
    fp8.fp8_quantize_dscale(x, fmt, scale, q)
    torch.cuda.synchronize()
    a = oracle.amax(h)
    s = oracle.scale_from_amax(a, fmt)
    assert amax.item() == a and np.float32(scale.item()) == s
    want = oracle.quantize(h, fmt, s)
    got = q.cpu().numpy()
    assert np.array_equal(got, want), "%d bytes differ" % int((got != want).sum())


def test_fp8_instruction_adder_window_is_what_the_header_says():
    """Documents, through the public entry points, why two GEMM variants exist: a product 2^-j
    times the largest product of its run of 8 consecutive K survives in fp8_gemm for every j
    that fp32 can hold, and is dropped by the FP8 matrix-core instructions from j = 14 on;
    in another run of 8 it survives in both."""
    M = N = 256
    K = 128
    def pow2(e):                      # E4M3 code of 2^e, -9 <= e <= 8
        return oracle.encode(E4M3, 2.0 ** e)
    lost_f16, lost_mfma8_same, lost_mfma8_other = [], [], []
    for j in range(0, 24):
        e = 16 - j
        x = max(-9, min(8, e // 2))
        y = e - x
        for small_k, bucket in ((1, lost_mfma8_same), (9, lost_mfma8_other)):
            A = np.zeros((M, K), dtype=np.uint8)
            B = np.zeros((K, N), dtype=np.uint8)
            A[0, 0] = pow2(8); B[0, 0] = pow2(8)
            A[0, small_k] = pow2(x); B[small_k, 0] = pow2(y)
            want = 2.0 ** 16 + 2.0 ** e
            S, _ = oracle.gemm_points(A, E4M3, B, E4M3, [0], [0])
            assert S[0] == want
            c16 = out_to_f64(run_gemm(A, E4M3, 1.0, B, E4M3, 1.0, fp8.FP8_F32))[0, 0]
            c8 = out_to_f64(run_gemm(A, E4M3, 1.0, B, E4M3, 1.0, fp8.FP8_F32, mode="mfma8"))[0, 0]
            if c16 != want and small_k == 1:
                lost_f16.append(j)
            if c8 != want:
                bucket.append(j)
            assert abs(c8 - want) <= 2.0 ** -10 * (2.0 ** 16 + 2.0 ** e)     # its documented bound
    assert lost_f16 == []
    assert lost_mfma8_other == []
    print("FP8 instructions drop the smaller product of a run of 8 for j in", lost_mfma8_same)
    assert lost_mfma8_same == list(range(14, 24))


# ---- operand storage orders (forward with out x in weights, dgrad, wgrad) ---------------------------

@pytest.fixture(params=["256", "128"])
def tile_n(request):
    """Both tile widths of the tiled kernel, whatever the dispatcher would choose."""
    old = fp8.fp8_set_knob(fp8.FP8_KNOB_TILE_N, int(request.param))
    yield request.param
    fp8.fp8_set_knob(fp8.FP8_KNOB_TILE_N, old)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_operand_layouts(transA, transB, mode, tile_n):
    """C = op(A) op(B) with either operand given transposed; tiled kernel shape and a ragged one."""
    rng = np.random.default_rng(50 + 2 * transA + transB)
    for (M, N, K) in [(512, 256, 640), (256, 512, 128), (100, 36, 72)]:
        A = random_codes(rng, (M, K), E5M2, 0x5F)
        B = random_codes(rng, (K, N), E4M3)
        S, T = oracle.gemm_rows(A, E5M2, B, E4M3)
        dA = to_dev(np.ascontiguousarray(A.T) if transA else A)
        dB = to_dev(np.ascontiguousarray(B.T) if transB else B)
        sA, sB = np.float32(1.7), np.float32(0.3)
        for out_dtype in (fp8.FP8_F32, fp8.FP8_BF16):
            C = torch.empty((M, N), dtype=OUT[out_dtype], device="cuda")
            fp8.fp8_gemm_ex(dA, E5M2, transA, dB, E4M3, transB, C, float(sA), float(sB),
                            fp8.FP8_GEMM_MFMA8 if mode == "mfma8" else 0)
            torch.cuda.synchronize()
            check(out_to_f64(C), S, T, sA, sB, out_dtype, "layout %d%d %s" % (transA, transB, (M, N, K)), mode=mode)
        # device scales
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        fp8.fp8_gemm_ex(dA, E5M2, transA, dB, E4M3, transB, C,
                        torch.tensor([sA], device="cuda"), torch.tensor([sB], device="cuda"),
                        fp8.FP8_GEMM_MFMA8 if mode == "mfma8" else 0)
        torch.cuda.synchronize()
        check(out_to_f64(C), S, T, sA, sB, fp8.FP8_F32, "layout, device scales", mode=mode)


@pytest.mark.parametrize("transA,transB", [(0, 1), (1, 0), (1, 1)])
def test_operand_layouts_exact_integers_long_k(transA, transB, tile_n):
    """Exact-integer operands over many stages (odd and even stage pairs, ring wrap-around)."""
    M, N, K = 256, 256, 128 * 13
    rng = np.random.default_rng(9 + transA)
    ai = rng.integers(-4, 5, (M, K)).astype(np.float32)
    bi = rng.integers(-4, 5, (K, N)).astype(np.float32)
    Aq, Bq = oracle.quantize(ai, E4M3, 1.0), oracle.quantize(bi, E4M3, 1.0)
    S, _ = oracle.gemm_rows(Aq, E4M3, Bq, E4M3)
    dA = to_dev(np.ascontiguousarray(Aq.T) if transA else Aq)
    dB = to_dev(np.ascontiguousarray(Bq.T) if transB else Bq)
    for flags in (0, fp8.FP8_GEMM_MFMA8):
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        fp8.fp8_gemm_ex(dA, E4M3, transA, dB, E4M3, transB, C, 1.0, 1.0, flags)
        torch.cuda.synchronize()
        assert np.array_equal(out_to_f64(C), S), (transA, transB, flags)


def test_training_step_gemms_of_a_linear_layer():
    """Forward, dgrad and wgrad of one linear layer from the same three FP8 tensors, no copies:
    X [tokens x in] E4M3, W [out x in] E4M3, dY [tokens x out] E5M2 (Section 3: formats by role)."""
    tokens, d_in, d_out = 512, 256, 768
    rng = np.random.default_rng(77)
    X = random_codes(rng, (tokens, d_in), E4M3)
    W = random_codes(rng, (d_out, d_in), E4M3)
    dY = random_codes(rng, (tokens, d_out), E5M2, 0x5F)
    dX_, dW_, dYd = to_dev(X), to_dev(W), to_dev(dY)
    Y = torch.empty((tokens, d_out), dtype=torch.bfloat16, device="cuda")
    dXo = torch.empty((tokens, d_in), dtype=torch.bfloat16, device="cuda")
    dWo = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    fp8.fp8_gemm_ex(dX_, E4M3, 0, dW_, E4M3, 1, Y, 2.0, 4.0)              # Y = X W^T
    fp8.fp8_gemm_ex(dYd, E5M2, 0, dW_, E4M3, 0, dXo, 8.0, 4.0)           # dX = dY W
    fp8.fp8_gemm_ex(dYd, E5M2, 1, dX_, E4M3, 0, dWo, 8.0, 2.0)           # dW = dY^T X
    torch.cuda.synchronize()
    S, T = oracle.gemm_rows(X, E4M3, np.ascontiguousarray(W.T), E4M3)
    check(out_to_f64(Y), S, T, 2.0, 4.0, fp8.FP8_BF16, "forward")
    S, T = oracle.gemm_rows(dY, E5M2, W, E4M3)
    check(out_to_f64(dXo), S, T, 8.0, 4.0, fp8.FP8_BF16, "dgrad")
    S, T = oracle.gemm_rows(np.ascontiguousarray(dY.T), E5M2, X, E4M3)
    check(out_to_f64(dWo), S, T, 8.0, 2.0, fp8.FP8_F32, "wgrad")


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_every_stage_count_through_the_loop_regions(transA, transB, mode, tile_n):
    """K from 1 to 41 stages of 64, and lengths that end inside a stage: the tiled kernel's K loop
    has a prologue, a steady-state region without load tests, a tested tail and a peeled last step;
    every length must hand over between them correctly (a wrong wait count or ring slot shows as a
    wrong sum), and a last stage pair that reaches beyond K must contribute zeros for the part
    beyond.  Integer operands: exact.  The operands sit at the very end of their allocations'
    used part and are followed by bytes that would show up in the sums if they were read."""
    rng = np.random.default_rng(70 + 2 * transA + transB)
    M, N = 256, 384
    def guarded(h):
        """h on the device, followed directly by 4 KB of the byte 0x7E (448 as E4M3)."""
        buf = torch.full((h.size + 4096,), 0x7E, dtype=torch.uint8, device="cuda")
        buf[:h.size] = torch.from_numpy(np.ascontiguousarray(h).reshape(-1)).cuda()
        return buf[:h.size].view(h.shape)
    for K in [64 * i for i in range(1, 42)] + [16, 48, 80, 144, 1936]:
        ai = rng.integers(-4, 5, (M, K)).astype(np.float32)
        bi = rng.integers(-4, 5, (K, N)).astype(np.float32)
        Aq, Bq = oracle.quantize(ai, E4M3, 1.0), oracle.quantize(bi, E4M3, 1.0)
        want = ai.astype(np.float64) @ bi.astype(np.float64)          # integers: exact in fp64 and in fp32
        dA = guarded(np.ascontiguousarray(Aq.T) if transA else Aq)
        dB = guarded(np.ascontiguousarray(Bq.T) if transB else Bq)
        C = torch.full((M, N), 7.0, dtype=torch.float32, device="cuda")
        assert fp8.fp8_gemm_plan(dA, transA, dB, transB, C) in TILED, K
        fp8.fp8_gemm_ex(dA, E4M3, transA, dB, E4M3, transB, C, 1.0, 1.0, fp8.FP8_GEMM_MFMA8 if mode == "mfma8" else 0)
        torch.cuda.synchronize()
        got = out_to_f64(C)
        assert np.array_equal(got, want), "K=%d layout %d%d %s tile %s: %d outputs differ" % (
            K, transA, transB, mode, tile_n, np.count_nonzero(got != want))


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_repeated_launches_give_identical_bits_while_memory_is_busy(transA, transB, mode, tile_n):
    """The tiled kernel tracks its direct global->LDS loads with hand-counted waits; a count that is
    one too lenient would read a slab before it has landed, but only when the memory system is slow
    enough.  25 launches of a 32-tile problem, each racing a large copy on a second stream, must all
    give the bits of the first launch (which is checked against the oracle)."""
    rng = np.random.default_rng(90 + 2 * transA + transB)
    M, N, K = 1024, 2048, 4096
    A, B = random_codes(rng, (M, K), E5M2, 0x6F), random_codes(rng, (K, N), E4M3)
    dA = to_dev(np.ascontiguousarray(A.T) if transA else A)
    dB = to_dev(np.ascontiguousarray(B.T) if transB else B)
    flags = fp8.FP8_GEMM_MFMA8 if mode == "mfma8" else 0
    C0 = torch.empty((M, N), dtype=torch.float32, device="cuda")
    fp8.fp8_gemm_ex(dA, E5M2, transA, dB, E4M3, transB, C0, 1.0, 1.0, flags)
    torch.cuda.synchronize()
    rows = np.array([0, 255, 256, 700, M - 1])
    S, T = oracle.gemm_rows(A, E5M2, B, E4M3, rows)
    check(out_to_f64(C0[torch.from_numpy(rows).cuda()]), S, T, np.float32(1.0), np.float32(1.0), fp8.FP8_F32,
          "first launch", mode=mode)
    src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    side = torch.cuda.Stream()
    C = torch.empty_like(C0)
    for rep in range(25):
        with torch.cuda.stream(side):
            dst.copy_(src, non_blocking=True)
        C.fill_(float(rep))
        fp8.fp8_gemm_ex(dA, E5M2, transA, dB, E4M3, transB, C, 1.0, 1.0, flags)
        torch.cuda.synchronize()
        assert torch.equal(C, C0), "launch %d differs from the first in %d outputs" % (rep, int((C != C0).sum()))


# ---- both tile widths in one launch --------------------------------------------------------------------

@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_mixed_tile_widths_exact_integers(transA, transB, mode):
    """256-wide tiles for the first columns and 128-wide ones for the rest, one launch (forced by the
    knob, and chosen by the dispatcher's model where it predicts a gain).  Shapes with a single wide
    column and many, with edge tiles in M and in N, with N that is no multiple of 16 (element-wise
    stores) and a K tail; integer operands, so the result must equal the oracle's exactly; nothing
    may be written outside C."""
    rng = np.random.default_rng(500 + 2 * transA + transB)
    shapes = [(512, 384, 256), (304, 1300 if transB else 1296, 448), (1024, 2048 + 128, 128), (256, 520 if transB else 528, 64), (720, 1000 if transB else 1008, 192)]
    for (M, N, K) in shapes:
        ai = rng.integers(-4, 5, (M, K)).astype(np.float32)
        bi = rng.integers(-4, 5, (K, N)).astype(np.float32)
        Aq, Bq = oracle.quantize(ai, E4M3, 1.0), oracle.quantize(bi, E5M2, 1.0)
        want = (ai.astype(np.float64) @ bi.astype(np.float64)) * 4.0
        dA = to_dev(np.ascontiguousarray(Aq.T) if transA else Aq)
        dB = to_dev(np.ascontiguousarray(Bq.T) if transB else Bq)
        for out_dtype in (fp8.FP8_F32, fp8.FP8_BF16):
            guard = 64
            flat = torch.full((M * N + 2 * guard,), 9.0, dtype=OUT[out_dtype], device="cuda")
            C = flat[guard:guard + M * N].view(M, N)
            with knob(fp8.FP8_KNOB_MIXED, 2):
                assert fp8.fp8_gemm_plan(dA, transA, dB, transB, C) & 15 == fp8.FP8_PLAN_TILED_MIXED, (M, N, K)
                fp8.fp8_gemm_ex(dA, E4M3, transA, dB, E5M2, transB, C, 0.5, 0.5, fp8.FP8_GEMM_MFMA8 if mode == "mfma8" else 0)
            torch.cuda.synchronize()
            ref = want if out_dtype == fp8.FP8_F32 else torch.from_numpy(want).to(torch.bfloat16).double().numpy()
            assert np.array_equal(out_to_f64(C), ref), "%s layout %d%d %s: %d outputs differ" % (
                (M, N, K), transA, transB, mode, np.count_nonzero(out_to_f64(C) != ref))
            assert torch.all(flat[:guard] == 9.0) and torch.all(flat[guard + M * N:] == 9.0), "wrote outside C"


@pytest.mark.parametrize("mode", MODES)
def test_mixed_tile_widths_chosen_by_the_dispatcher_and_within_the_bound(mode):
    """The dispatcher picks the mixed launch by itself for 4096 x 6144 with a long K (384 wide tiles =
    1.5 rounds of the chip); random codes against the oracle on sampled rows, and the same bits as
    the single-width launches give (every output accumulates its K in the same order whatever the tile)."""
    rng = np.random.default_rng(77)
    M, N, K = 4096, 6144, 8192
    A, B = random_codes(rng, (M, K), E4M3), random_codes(rng, (K, N), E4M3)
    rows = np.sort(rng.choice(M, 24, replace=False))
    S, T = oracle.gemm_rows(A, E4M3, B, E4M3, rows)
    dA, dB = to_dev(A), to_dev(B)
    flags = fp8.FP8_GEMM_MFMA8 if mode == "mfma8" else 0
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    assert fp8.fp8_gemm_plan(dA, 0, dB, 0, C) == fp8.FP8_PLAN_TILED_MIXED
    fp8.fp8_gemm_ex(dA, E4M3, 0, dB, E4M3, 0, C, 2.0, 3.0, flags)
    torch.cuda.synchronize()
    check(out_to_f64(C[torch.from_numpy(rows).cuda()]), S, T, 2.0, 3.0, fp8.FP8_F32, "mixed widths", mode=mode)
    for tile in (128, 256):
        C1 = torch.empty((M, N), dtype=torch.float32, device="cuda")
        with knob(fp8.FP8_KNOB_TILE_N, tile), knob(fp8.FP8_KNOB_PERSIST, 1):
            fp8.fp8_gemm_ex(dA, E4M3, 0, dB, E4M3, 0, C1, 2.0, 3.0, flags)
        torch.cuda.synchronize()
        assert torch.equal(C, C1), "mixed and %d-wide launches differ" % tile


# ---- the persistent form of the narrow tile ---------------------------------------------------------

@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_persistent_form_exact_integers_over_tile_sequences(transA, transB, mode):
    """One workgroup per compute unit walks several 256 x 128 tiles as one K loop (loads of the next
    tile issued during the current one, outputs stored straight from the registers).  Integer
    operands (exact sums) over shapes that give the workgroups one, two and three tiles each, from the
    shortest K the form takes (8 stages) on, fp32 and bf16 outputs; the result must also equal the
    one-workgroup-per-tile kernel's bit for bit."""
    rng = np.random.default_rng(300 + 2 * transA + transB)
    flags = fp8.FP8_GEMM_MFMA8 if mode == "mfma8" else 0
    for (M, N, K) in [(1024, 9216, 512), (2048, 5120, 640), (4096, 6144, 512), (1024, 9216, 1152), (256, 128 * 5, 2048)]:
        ai = rng.integers(-4, 5, (M, K)).astype(np.float32)
        bi = rng.integers(-4, 5, (K, N)).astype(np.float32)
        Aq, Bq = oracle.quantize(ai, E4M3, 1.0), oracle.quantize(bi, E4M3, 1.0)
        want = (ai.astype(np.float64) @ bi.astype(np.float64)) * 0.5
        dA = to_dev(np.ascontiguousarray(Aq.T) if transA else Aq)
        dB = to_dev(np.ascontiguousarray(Bq.T) if transB else Bq)
        for out_dtype in (fp8.FP8_F32, fp8.FP8_BF16):
            C = torch.full((M, N), 7.0, dtype=OUT[out_dtype], device="cuda")
            with knob(fp8.FP8_KNOB_PERSIST, 2), knob(fp8.FP8_KNOB_TILE_N, 128):
                assert fp8.fp8_gemm_plan(dA, transA, dB, transB, C) == fp8.FP8_PLAN_TILED_256x128 | fp8.FP8_PLAN_PERSISTENT
                fp8.fp8_gemm_ex(dA, E4M3, transA, dB, E4M3, transB, C, 2.0, 1.0, flags)
            C1 = torch.full((M, N), 8.0, dtype=OUT[out_dtype], device="cuda")
            with knob(fp8.FP8_KNOB_PERSIST, 1), knob(fp8.FP8_KNOB_TILE_N, 128):
                assert fp8.fp8_gemm_plan(dA, transA, dB, transB, C1) == fp8.FP8_PLAN_TILED_256x128
                fp8.fp8_gemm_ex(dA, E4M3, transA, dB, E4M3, transB, C1, 2.0, 1.0, flags)
            torch.cuda.synchronize()
            assert torch.equal(C, C1), "persistent and per-tile kernels differ: %s" % ((M, N, K, out_dtype),)
            got = out_to_f64(C)
            ref = want if out_dtype == fp8.FP8_F32 else torch.from_numpy(want).to(torch.bfloat16).double().numpy()
            assert np.array_equal(got, ref), "%s layout %d%d %s: %d outputs differ" % (
                (M, N, K), transA, transB, mode, np.count_nonzero(got != ref))


@pytest.mark.parametrize("mode", MODES)
def test_persistent_form_random_codes_within_the_bound_and_repeatable(mode):
    rng = np.random.default_rng(311)
    M, N, K = 2048, 5120, 1024
    A, B = random_codes(rng, (M, K), E5M2, 0x5F), random_codes(rng, (K, N), E4M3)
    dA, dB = to_dev(A), to_dev(B)
    flags = fp8.FP8_GEMM_MFMA8 if mode == "mfma8" else 0
    sA, sB = np.float32(2.5), np.float32(0.125)
    with knob(fp8.FP8_KNOB_PERSIST, 2), knob(fp8.FP8_KNOB_TILE_N, 128):
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        fp8.fp8_gemm_ex(dA, E5M2, 0, dB, E4M3, 0, C, float(sA), float(sB), flags)
        C2 = torch.empty_like(C)
        fp8.fp8_gemm_ex(dA, E5M2, 0, dB, E4M3, 0, C2, torch.tensor([sA], device="cuda"), torch.tensor([sB], device="cuda"), flags)
    torch.cuda.synchronize()
    assert torch.equal(C, C2)
    rows = np.array([0, 255, 256, 1000, M - 1])
    S, T = oracle.gemm_rows(A, E5M2, B, E4M3, rows)
    check(out_to_f64(C[torch.from_numpy(rows).cuda()]), S, T, sA, sB, fp8.FP8_F32, "persistent form", mode=mode)
    w = freivalds_blocks(C, A, E5M2, B, E4M3, sA, sB, oracle.F32, rel=REL[mode], block=128, label="persistent form")
    print("persistent form %s: block sums worst err/bound %.3f" % (mode, w), flush=True)
