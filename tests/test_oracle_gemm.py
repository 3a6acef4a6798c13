"""Pins for the oracle's GEMM reference and acceptance bound."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import E4M3, E5M2, F32, BF16

FMTS = [E4M3, E5M2]


def finite_codes(fmt):
    v = oracle.decode_all(fmt)
    return np.flatnonzero(np.isfinite(v)).astype(np.uint8)


def random_fp8(rng, shape, fmt):
    return rng.choice(finite_codes(fmt), size=shape).astype(np.uint8)


@pytest.mark.parametrize("fmtA,fmtB", [(E4M3, E4M3), (E5M2, E4M3), (E4M3, E5M2), (E5M2, E5M2)])
def test_tiny_shapes_against_exact_rational_triple_loop(fmtA, fmtB):
    rng = np.random.default_rng(42 + 2 * fmtA + fmtB)
    va = [Fraction(x) if np.isfinite(x) else None for x in oracle.decode_all(fmtA)]
    vb = [Fraction(x) if np.isfinite(x) else None for x in oracle.decode_all(fmtB)]
    for (M, N, K) in [(1, 1, 1), (2, 3, 5), (4, 2, 7), (3, 5, 8), (8, 8, 8)]:
        A = random_fp8(rng, (M, K), fmtA)
        B = random_fp8(rng, (K, N), fmtB)
        S, T = oracle.gemm_rows(A, fmtA, B, fmtB)
        for i in range(M):
            for j in range(N):
                s = sum(va[A[i, k]] * vb[B[k, j]] for k in range(K))
                t = sum(abs(va[A[i, k]] * vb[B[k, j]]) for k in range(K))
                # the exact sums need < 53 bits here only sometimes: compare within fp64 rounding
                assert abs(Fraction(S[i, j]) - s) <= Fraction(2) ** -50 * t
                assert abs(Fraction(T[i, j]) - t) <= Fraction(2) ** -50 * t


@pytest.mark.parametrize("fmt", FMTS)
def test_every_byte_pattern_as_operand(fmt):
    """A holds all finite codes once per row; B is an identity: S must be decode(A)."""
    codes = finite_codes(fmt)
    K = codes.size
    A = np.stack([codes, codes[::-1]])
    one = oracle.encode(E4M3, 1.0)
    B = np.zeros((K, K), dtype=np.uint8)
    B[np.arange(K), np.arange(K)] = one
    S, T = oracle.gemm_rows(A, fmt, B, E4M3)
    want = oracle.decode_all(fmt)[A]
    assert np.array_equal(S, want)
    assert np.array_equal(T, np.abs(want))


def test_transposed_operand_would_be_noticed():
    """A one-hot probe fixes which index of B is the reduction index (B is K x N)."""
    M, N, K = 3, 4, 5
    A = np.zeros((M, K), dtype=np.uint8)
    B = np.zeros((K, N), dtype=np.uint8)
    A[1, 3] = oracle.encode(E4M3, 2.0)
    B[3, 2] = oracle.encode(E4M3, -3.0)
    B[2, 3] = oracle.encode(E4M3, 5.0)
    S, T = oracle.gemm_rows(A, E4M3, B, E4M3)
    want = np.zeros((M, N))
    want[1, 2] = -6.0
    assert np.array_equal(S, want)
    assert np.array_equal(T, np.abs(want))


@pytest.mark.parametrize("fmtA,fmtB", [(E4M3, E4M3), (E5M2, E4M3)])
def test_against_fp64_blas(fmtA, fmtB):
    """Library cross-check: torch's fp64 matmul of the decoded operands."""
    rng = np.random.default_rng(5)
    M, N, K = 37, 53, 300
    A = random_fp8(rng, (M, K), fmtA)
    B = random_fp8(rng, (K, N), fmtB)
    da = torch.from_numpy(oracle.decode_all(fmtA)[A])
    db = torch.from_numpy(oracle.decode_all(fmtB)[B])
    S, T = oracle.gemm_rows(A, fmtA, B, fmtB)
    lib_S = (da @ db).numpy()
    lib_T = (da.abs() @ db.abs()).numpy()
    assert np.all(np.abs(S - lib_S) <= 1e-13 * lib_T)
    assert np.all(np.abs(T - lib_T) <= 1e-13 * lib_T)


def test_points_equal_rows():
    rng = np.random.default_rng(8)
    M, N, K = 19, 23, 129
    A = random_fp8(rng, (M, K), E5M2)
    B = random_fp8(rng, (K, N), E4M3)
    S, T = oracle.gemm_rows(A, E5M2, B, E4M3)
    pi = rng.integers(0, M, 200)
    pj = rng.integers(0, N, 200)
    Sp, Tp = oracle.gemm_points(A, E5M2, B, E4M3, pi, pj)
    assert np.array_equal(Sp, S[pi, pj]) and np.array_equal(Tp, T[pi, pj])
    Sr, Tr = oracle.gemm_rows(A, E5M2, B, E4M3, rows=[18, 0, 7])
    assert np.array_equal(Sr, S[[18, 0, 7]]) and np.array_equal(Tr, T[[18, 0, 7]])


def test_small_integer_operands_are_exact():
    """Integers up to 16 are exact in E4M3; sums stay far below 2^53."""
    rng = np.random.default_rng(21)
    M, N, K = 16, 16, 512
    ai = rng.integers(-8, 9, (M, K))
    bi = rng.integers(-8, 9, (K, N))
    A = oracle.quantize(ai.astype(np.float32), E4M3, 1.0)
    B = oracle.quantize(bi.astype(np.float32), E4M3, 1.0)
    S, T = oracle.gemm_rows(A, E4M3, B, E4M3)
    assert np.array_equal(S, (ai @ bi).astype(np.float64))
    assert np.array_equal(T, (np.abs(ai) @ np.abs(bi)).astype(np.float64))


def test_non_finite_operands_follow_ieee():
    A = np.array([[oracle.encode(E5M2, np.inf), oracle.encode(E5M2, 1.0)]], dtype=np.uint8)
    B = np.array([[oracle.encode(E4M3, 2.0)], [oracle.encode(E4M3, np.nan)]], dtype=np.uint8)
    S, _ = oracle.gemm_rows(A, E5M2, B, E4M3)
    assert np.isnan(S[0, 0])
    B[1, 0] = oracle.encode(E4M3, 1.0)
    S, _ = oracle.gemm_rows(A, E5M2, B, E4M3)
    assert S[0, 0] == np.inf


def test_unscale_and_bound():
    S = np.array([3.0, -1.0, 0.0, 1000.0])
    T = np.array([5.0, 1.0, 0.0, 1000.0])
    sA, sB = np.float32(4.0), np.float32(0.5)
    c, bound = oracle.gemm_bound(S, T, sA, sB, F32)
    assert np.array_equal(c, S / 2.0)
    # ulp pins: numpy's spacing for float32; 2^-7 relative step for bfloat16
    half_ulp = 0.5 * np.spacing(np.abs(c).astype(np.float32)).astype(np.float64)
    want = 2.0 ** -20 * T / 2.0 + half_ulp
    nz = c != 0
    assert np.array_equal(bound[nz], want[nz])
    _, bound16 = oracle.gemm_bound(S, T, sA, sB, BF16)
    assert bound16[0] == 2.0 ** -20 * 2.5 + 0.5 * 2.0 ** (0 - 7)     # c = 1.5, e = 0
    assert bound16[3] == 2.0 ** -20 * 500.0 + 0.5 * 2.0 ** (8 - 7)   # c = 500, e = 8
    # arbitrary (non power of two) scales: alpha is the fp64 reciprocal of the fp32 product
    sA, sB = np.float32(0.1), np.float32(3.3)
    c, _ = oracle.gemm_bound(S, T, sA, sB, F32)
    assert np.allclose(c, S / (float(sA) * float(sB)), rtol=1e-15)


def test_ulp_matches_library_spacing():
    rng = np.random.default_rng(2)
    c = (rng.standard_normal(5000) * 2.0 ** rng.integers(-100, 100, 5000))
    c32 = c.astype(np.float32).astype(np.float64)
    assert np.array_equal(oracle.ulp(c32, F32), np.spacing(np.abs(c32).astype(np.float32)).astype(np.float64))
    # bfloat16: spacing from torch.nextafter-free construction: bits + 1
    t = torch.from_numpy(c.astype(np.float32)).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16).astype(np.uint32)
    lo = ((bits & 0x7FFF) << 16).view(np.float32).astype(np.float64)
    hi = (((bits & 0x7FFF) + 1) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(oracle.ulp(lo, BF16), hi - lo)


def test_unscale_channels_is_row_and_column_scaling_of_the_operands():
    """Per-channel factors taken out after the product equal the product of operands that were
    divided by them first (a diagonal matrix commutes out of a matrix product); power-of-two
    factors make both sides exact, so the identity is checked bit for bit against numpy's matmul."""
    rng = np.random.default_rng(5)
    M, N, K = 7, 9, 24
    A = rng.integers(0, 0x60, (M, K)).astype(np.uint8) | (rng.integers(0, 2, (M, K)).astype(np.uint8) << 7)
    B = rng.integers(0, 0x60, (K, N)).astype(np.uint8) | (rng.integers(0, 2, (K, N)).astype(np.uint8) << 7)
    sA = np.ldexp(1.0, rng.integers(-6, 7, M)).astype(np.float32)
    sB = np.ldexp(1.0, rng.integers(-6, 7, N)).astype(np.float32)
    S, T = oracle.gemm_rows(A, E4M3, B, E4M3)
    c, alpha = oracle.unscale_channels(S, sA, sB)
    dec = oracle.decode_all(E4M3)
    want = (dec[A] / sA[:, None].astype(np.float64)) @ (dec[B] / sB[None, :].astype(np.float64))
    assert np.array_equal(c, want)
    assert np.array_equal(alpha, 1.0 / np.outer(sA.astype(np.float64), sB.astype(np.float64)))
    # one value per tensor is the special case of constant vectors, and equals unscale()
    c1, _ = oracle.unscale_channels(S, np.float32(0.3), np.float32(7.0))
    c2, _ = oracle.unscale_channels(S, np.full(M, 0.3, np.float32), np.full(N, 7.0, np.float32))
    c3, _ = oracle.unscale(S, np.float32(0.3), np.float32(7.0))
    assert np.array_equal(c1, c2) and np.allclose(c1, c3, rtol=1e-15)
    # a transposed or swapped use of the vectors is noticed
    with pytest.raises(ValueError):
        oracle.unscale_channels(S, sB, sA)
    # bound with vectors: 2^-20 * alpha_ij * T_ij + ulp/2
    _, bound = oracle.gemm_bound(S, T, sA, sB, F32)
    assert np.allclose(bound, 2.0 ** -20 * alpha * T + 0.5 * oracle.ulp(c, F32), rtol=1e-15)


def test_block_sums_equal_the_blockwise_sums_of_the_row_reference():
    """gemm_block_sums (the whole-matrix check of the large workloads) against the plain
    definition: S and T of every output from gemm_rows, multiplied by r and added up block by block
    with Python loops; ragged last block, both signs, all four format mixes."""
    rng = np.random.default_rng(41)
    M, N, K, block = 9, 23, 37, 5
    for fmtA in (oracle.E4M3, oracle.E5M2):
        for fmtB in (oracle.E4M3, oracle.E5M2):
            A = rng.integers(0, 0x70 if fmtA == oracle.E4M3 else 0x60, (M, K)).astype(np.uint8) | \
                (rng.integers(0, 2, (M, K)).astype(np.uint8) << 7)
            B = rng.integers(0, 0x70 if fmtB == oracle.E4M3 else 0x60, (K, N)).astype(np.uint8) | \
                (rng.integers(0, 2, (K, N)).astype(np.uint8) << 7)
            r = rng.choice([-1.0, 1.0], N)
            S, T = oracle.gemm_rows(A, fmtA, B, fmtB)
            SR, TR = oracle.gemm_block_sums(A, fmtA, B, fmtB, r, block)
            nb = (N + block - 1) // block
            assert SR.shape == (M, nb) and TR.shape == (M, nb)
            for i in range(M):
                for t in range(nb):
                    want_s = sum(r[j] * S[i, j] for j in range(t * block, min(N, (t + 1) * block)))
                    want_t = sum(T[i, j] for j in range(t * block, min(N, (t + 1) * block)))
                    assert abs(SR[i, t] - want_s) <= 1e-12 * want_t + 1e-300
                    assert abs(TR[i, t] - want_t) <= 1e-12 * want_t + 1e-300
    with pytest.raises(ValueError):
        oracle.gemm_block_sums(np.full((2, 2), 0x7F, np.uint8), oracle.E4M3, np.zeros((2, 2), np.uint8), oracle.E4M3, [1, 1], 2)
