"""CPU oracle for the scaled-FP8 matrix multiply path -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes access to ``fp8_oracle.c`` (plain C, written from Table 1 and
Sections 2-3 of "FP8 Formats for Deep Learning", arXiv 2209.05433) plus the
acceptance bound for the GEMM.  Only ``tests/``, the smoke check and the bench's
``cpu_baseline`` leg may import this package; the HIP library and its Python
binding never do, and nothing here imports them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

E4M3, E5M2 = 0, 1
F32, BF16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fp8_oracle.c")
_LIB = os.path.join(_HERE, "libfp8oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (IEEE semantics: no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    c = ctypes
    lib.fp8o_decode.restype = c.c_double
    lib.fp8o_decode.argtypes = [c.c_int, c.c_uint8]
    lib.fp8o_encode.restype = c.c_uint8
    lib.fp8o_encode.argtypes = [c.c_int, c.c_float, c.c_int]
    lib.fp8o_amax.restype = c.c_float
    lib.fp8o_amax.argtypes = [c.c_void_p, c.c_size_t, c.c_int]
    lib.fp8o_scale_from_amax.restype = c.c_float
    lib.fp8o_scale_from_amax.argtypes = [c.c_float, c.c_int]
    lib.fp8o_quantize.restype = None
    lib.fp8o_quantize.argtypes = [c.c_void_p, c.c_size_t, c.c_int, c.c_int, c.c_float,
                                  c.c_int, c.c_void_p]
    lib.fp8o_dequantize.restype = None
    lib.fp8o_dequantize.argtypes = [c.c_void_p, c.c_size_t, c.c_int, c.c_float, c.c_void_p]
    lib.fp8o_gemm_points.restype = None
    lib.fp8o_gemm_points.argtypes = [c.c_void_p, c.c_int, c.c_void_p, c.c_int,
                                     c.c_int64, c.c_int64, c.c_int64,
                                     c.c_void_p, c.c_void_p, c.c_int64,
                                     c.c_void_p, c.c_void_p]
    lib.fp8o_gemm_rows.restype = None
    lib.fp8o_gemm_rows.argtypes = [c.c_void_p, c.c_int, c.c_void_p, c.c_int,
                                   c.c_int64, c.c_int64, c.c_int64,
                                   c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p]
    lib.fp8o_gemm_block_sums.restype = c.c_int
    lib.fp8o_gemm_block_sums.argtypes = [c.c_void_p, c.c_int, c.c_void_p, c.c_int, c.c_int64, c.c_int64, c.c_int64,
                                         c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.fp8o_encode_sr.restype = c.c_uint8
    lib.fp8o_encode_sr.argtypes = [c.c_int, c.c_float, c.c_uint32]
    lib.fp8o_philox4x32.restype = None
    lib.fp8o_philox4x32.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p]
    lib.fp8o_sr_bits.restype = c.c_uint32
    lib.fp8o_sr_bits.argtypes = [c.c_uint64, c.c_uint64]
    lib.fp8o_quantize_sr.restype = None
    lib.fp8o_quantize_sr.argtypes = [c.c_void_p, c.c_size_t, c.c_int, c.c_int, c.c_float, c.c_uint64, c.c_void_p]
    lib.fp8o_num_threads.restype = c.c_int
    lib.fp8o_num_threads.argtypes = []
    _lib = lib
    return lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _as_input(x: np.ndarray):
    """float32 arrays are F32; uint16 arrays hold bfloat16 bit patterns."""
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        return x, F32
    if x.dtype == np.uint16:
        return x, BF16
    raise TypeError("oracle inputs are float32 or uint16 (bfloat16 bits), got %s" % x.dtype)


def num_threads() -> int:
    return int(_load().fp8o_num_threads())


def decode(fmt: int, b: int) -> float:
    return float(_load().fp8o_decode(fmt, int(b) & 0xFF))


def decode_all(fmt: int) -> np.ndarray:
    """decode() of the 256 byte values, as float64."""
    return np.array([decode(fmt, b) for b in range(256)], dtype=np.float64)


def encode(fmt: int, y, saturating: bool = True) -> int:
    return int(_load().fp8o_encode(fmt, float(np.float32(y)), int(saturating)))


def amax(x: np.ndarray) -> np.float32:
    x, dt = _as_input(x)
    return np.float32(_load().fp8o_amax(_ptr(x), x.size, dt))


def scale_from_amax(amax_value, fmt: int) -> np.float32:
    return np.float32(_load().fp8o_scale_from_amax(float(np.float32(amax_value)), fmt))


def quantize(x: np.ndarray, fmt: int, scale, saturating: bool = True) -> np.ndarray:
    x, dt = _as_input(x)
    q = np.empty(x.shape, dtype=np.uint8)
    _load().fp8o_quantize(_ptr(x), x.size, dt, fmt, float(np.float32(scale)),
                          int(saturating), _ptr(q))
    return q


def encode_sr(fmt: int, y, r16: int) -> int:
    """Stochastic rounding of one fp32 value with the 16 random bits r16."""
    return int(_load().fp8o_encode_sr(fmt, float(np.float32(y)), int(r16) & 0xFFFF))


def philox4x32(ctr, key) -> np.ndarray:
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    _load().fp8o_philox4x32(_ptr(c), _ptr(k), _ptr(out))
    return out


def sr_bits(seed: int, i: int) -> int:
    return int(_load().fp8o_sr_bits(int(seed), int(i)))


def quantize_sr(x: np.ndarray, fmt: int, scale, seed: int) -> np.ndarray:
    x, dt = _as_input(x)
    q = np.empty(x.shape, dtype=np.uint8)
    _load().fp8o_quantize_sr(_ptr(x), x.size, dt, fmt, float(np.float32(scale)), int(seed), _ptr(q))
    return q


def amax_rows(x: np.ndarray) -> np.ndarray:
    """amax of every row of a 2-D tensor: the per-tensor definition applied to each row on its own
    (per-channel granularity, Section 4.2)."""
    return np.array([amax(x[r]) for r in range(x.shape[0])], dtype=np.float32)


def scale_from_amax_n(amax_values, fmt: int) -> np.ndarray:
    return np.array([scale_from_amax(a, fmt) for a in np.asarray(amax_values, dtype=np.float32).reshape(-1)],
                    dtype=np.float32)


def quantize_rows(x: np.ndarray, fmt: int, scales, saturating: bool = True) -> np.ndarray:
    """Row r of a 2-D tensor quantized with its own scaling factor scales[r]."""
    scales = np.asarray(scales, dtype=np.float32).reshape(-1)
    if scales.size != x.shape[0]:
        raise ValueError("one scale per row expected")
    return np.stack([quantize(x[r], fmt, scales[r], saturating) for r in range(x.shape[0])]) if x.shape[0] else \
        np.empty(x.shape, dtype=np.uint8)


def scale_from_amax_history(history, fmt: int) -> np.float32:
    """Scaling factor from the largest of a list of earlier maxima (the maxima are magnitudes, so
    their amax is their maximum, NaN propagating); an empty history gives the factor 1."""
    h = np.ascontiguousarray(history, dtype=np.float32).reshape(-1)
    return scale_from_amax(amax(h) if h.size else np.float32(0.0), fmt)


def dequantize(q: np.ndarray, fmt: int, scale) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.uint8)
    out = np.empty(q.shape, dtype=np.float64)
    _load().fp8o_dequantize(_ptr(q), q.size, fmt, float(np.float32(scale)), _ptr(out))
    return out


def _check_ab(A, B):
    A = np.ascontiguousarray(A, dtype=np.uint8)
    B = np.ascontiguousarray(B, dtype=np.uint8)
    M, K = A.shape
    K2, N = B.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    return A, B, M, N, K


def gemm_points(A, fmtA, B, fmtB, pi, pj):
    """S and T (fp64 sum and sum of magnitudes of the products) at outputs (pi[p], pj[p])."""
    A, B, M, N, K = _check_ab(A, B)
    pi = np.ascontiguousarray(pi, dtype=np.int64)
    pj = np.ascontiguousarray(pj, dtype=np.int64)
    if pi.shape != pj.shape or (pi.size and (pi.min() < 0 or pi.max() >= M
                                              or pj.min() < 0 or pj.max() >= N)):
        raise ValueError("sample points out of range")
    S = np.empty(pi.shape, dtype=np.float64)
    T = np.empty(pi.shape, dtype=np.float64)
    _load().fp8o_gemm_points(_ptr(A), fmtA, _ptr(B), fmtB, M, N, K,
                             _ptr(pi), _ptr(pj), pi.size, _ptr(S), _ptr(T))
    return S, T


def gemm_rows(A, fmtA, B, fmtB, rows=None):
    """S and T for whole output rows (all rows when ``rows`` is None)."""
    A, B, M, N, K = _check_ab(A, B)
    rows = np.arange(M, dtype=np.int64) if rows is None else \
        np.ascontiguousarray(rows, dtype=np.int64)
    if rows.size and (rows.min() < 0 or rows.max() >= M):
        raise ValueError("row index out of range")
    S = np.empty((rows.size, N), dtype=np.float64)
    T = np.empty((rows.size, N), dtype=np.float64)
    _load().fp8o_gemm_rows(_ptr(A), fmtA, _ptr(B), fmtB, M, N, K,
                           _ptr(rows), rows.size, _ptr(S), _ptr(T))
    return S, T


def unscale(S, sA, sB):
    """C_ref = S / (sA*sB): the reciprocal of the two scales is applied once per
    dot product (Section 2, scaling paragraph), here in double precision."""
    alpha = 1.0 / (float(np.float32(sA)) * float(np.float32(sB)))
    return alpha * np.asarray(S, dtype=np.float64), alpha


def unscale_channels(S, sA, sB):
    """C_ref[i, j] = S[i, j] / (sA[i] * sB[j]) in double precision: per-channel scaling factors
    (Section 4.2 uses them for weights) taken out once per dot product.  sA: one value or one per
    row of S; sB: one value or one per column.  Returns (C_ref, alpha) with alpha[i, j] =
    1 / (sA[i] * sB[j]) broadcast to the shape of S."""
    S = np.asarray(S, dtype=np.float64)
    a = np.asarray(sA, dtype=np.float32).astype(np.float64).reshape(-1)
    b = np.asarray(sB, dtype=np.float32).astype(np.float64).reshape(-1)
    if a.size not in (1, S.shape[0]) or b.size not in (1, S.shape[1]):
        raise ValueError("scale vectors do not match the rows / columns of S")
    alpha = np.broadcast_to(1.0 / (a[:, None] * b[None, :]), S.shape)
    return alpha * S, alpha


def ulp(c_ref, out_dtype: int) -> np.ndarray:
    """Spacing of the output type at |c_ref|: 2^(e-23) for fp32, 2^(e-7) for
    bfloat16, e = floor(log2|c_ref|), clamped at the smallest normal exponent."""
    c = np.abs(np.asarray(c_ref, dtype=np.float64))
    _, e = np.frexp(c)                  # c = m * 2^e with m in [0.5, 1)
    e = np.maximum(e - 1, -126)         # floor(log2 c); zero and subnormals -> 2^-126 binade
    mant = 23 if out_dtype == F32 else 7
    return np.ldexp(1.0, e - mant)


def gemm_bound(S, T, sA, sB, out_dtype: int):
    """Reference value and acceptance bound for GEMM outputs:
    |C - C_ref| <= 2^-20 * alpha * T + ulp_out(C_ref)/2 with C_ref = alpha * S."""
    c_ref, alpha = unscale_channels(S, sA, sB) if (np.size(sA) > 1 or np.size(sB) > 1) else unscale(S, sA, sB)
    bound = 2.0 ** -20 * alpha * np.asarray(T, dtype=np.float64) + 0.5 * ulp(c_ref, out_dtype)
    return c_ref, bound


def gemm_block_sums(A, fmtA, B, fmtB, r, block: int):
    """Signed sums of the reference product over blocks of consecutive columns, in double precision:
        SR[i, t] = sum_{j in block t} r[j] * S[i, j],    TR[i, t] = sum_{j in block t} T[i, j]
    with S, T as in gemm_rows (sum and sum of magnitudes of the products a_ik b_kj over k), r one
    multiplier of magnitude 1 per column and block t = columns [t*block, (t+1)*block).  By linearity
    SR = dec(A) (dec(B) R) with R the N x nb matrix that holds r on its block pattern, which costs
    O(MK nb + KN) instead of O(MNK): the whole-matrix check for problems whose every output the plain
    loops cannot reach (a Freivalds check, one random sign vector per block of columns).  Finite
    operands only."""
    A, B, M, N, K = _check_ab(A, B)
    r = np.ascontiguousarray(r, dtype=np.float64).reshape(-1)
    if r.size != N or block <= 0 or not np.all(np.abs(r) == 1.0):
        raise ValueError("one multiplier of magnitude 1 per column and a positive block width expected")
    nb = (N + block - 1) // block
    BR = np.empty((K, nb), dtype=np.float64)
    BT = np.empty((K, nb), dtype=np.float64)
    SR = np.empty((M, nb), dtype=np.float64)
    TR = np.empty((M, nb), dtype=np.float64)
    if _load().fp8o_gemm_block_sums(_ptr(A), fmtA, _ptr(B), fmtB, M, N, K, _ptr(r), block,
                                    _ptr(BR), _ptr(BT), _ptr(SR), _ptr(TR)):
        raise ValueError("gemm_block_sums takes finite operands only")
    return SR, TR
