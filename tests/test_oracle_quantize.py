"""Pins for the oracle's amax, scale and scaled cast (Section 2, scaling paragraph)."""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import E4M3, E5M2
from workloads import synth

FMTS = [E4M3, E5M2]
MAXCODE = {E4M3: 0x7E, E5M2: 0x7B}
FMAX = {E4M3: 448.0, E5M2: 57344.0}
TORCH = {E4M3: torch.float8_e4m3fn, E5M2: torch.float8_e5m2}


def all_bf16_bits():
    return np.arange(65536, dtype=np.uint32).astype(np.uint16)


def test_amax_is_numpy_max_abs():
    x = synth.normal(300_001, 5)
    assert oracle.amax(x) == np.max(np.abs(x))
    h = synth.to_bf16_bits(x)
    assert oracle.amax(h) == np.max(np.abs(synth.bf16_bits_to_f32(h)))
    assert oracle.amax(np.zeros(0, dtype=np.float32)) == 0.0
    z = oracle.amax(np.array([-0.0], dtype=np.float32))
    assert z == 0.0 and not np.signbit(z)
    assert oracle.amax(np.array([1.0, -7.5, 3.0], dtype=np.float32)) == 7.5


def test_amax_specials():
    assert math.isnan(oracle.amax(np.array([1.0, np.nan, np.inf], dtype=np.float32)))
    assert oracle.amax(np.array([1.0, -np.inf], dtype=np.float32)) == np.inf
    # bf16: NaN bit pattern 0x7FC0, -inf 0xFF80
    assert math.isnan(oracle.amax(np.array([0x3F80, 0xFFC1], dtype=np.uint16)))
    assert oracle.amax(np.array([0x3F80, 0xFF80], dtype=np.uint16)) == np.inf


@pytest.mark.parametrize("fmt", FMTS)
def test_scale_maps_amax_to_format_max(fmt):
    rng = np.random.default_rng(3)
    for a in np.concatenate([2.0 ** rng.uniform(-30, 30, 2000),
                             [1.0, 448.0, 57344.0, 4567.0]]).astype(np.float32):
        s = oracle.scale_from_amax(a, fmt)
        assert s == np.float32(FMAX[fmt]) / np.float32(a)        # numpy's IEEE fp32 division
        assert oracle.quantize(np.array([a, -a], dtype=np.float32), fmt, s).tolist() == \
            [MAXCODE[fmt], 0x80 | MAXCODE[fmt]]
    for bad in (0.0, np.nan, np.inf, np.float32(1e-45)):     # quotient overflows for the last
        assert oracle.scale_from_amax(bad, fmt) == 1.0


@pytest.mark.parametrize("fmt", FMTS)
def test_power_of_two_scale_is_single_rounding(fmt):
    """With a power-of-two scale the fp32 product is exact, so the result must be the
    nearest FP8 value of the real product x*s: checked in exact rationals."""
    tab = [Fraction(oracle.decode(fmt, c)) for c in range(MAXCODE[fmt] + 1)]
    rng = np.random.default_rng(11 + fmt)
    x = (rng.standard_normal(3000) * 2.0 ** rng.integers(-6, 6, 3000)).astype(np.float32)
    for p in (-7, -1, 0, 3, 9):
        s = np.float32(2.0 ** p)
        q = oracle.quantize(x, fmt, s)
        for xi, qi in zip(x.tolist(), q.tolist()):
            m = abs(Fraction(xi)) * Fraction(2) ** p
            if m >= tab[-1]:
                want = len(tab) - 1
            else:
                d = [abs(m - v) for v in tab]
                dm = min(d)
                cands = [c for c, dv in enumerate(d) if dv == dm]
                want = [c for c in cands if c % 2 == 0][0] if len(cands) == 2 else cands[0]
            assert qi == (want | (0x80 if math.copysign(1, xi) < 0 else 0))


def test_product_is_rounded_to_single_precision_first():
    """A case where rounding the product to fp32 first changes the byte: the exact product
    lies just above an E4M3 midpoint, its fp32 rounding lands on the midpoint (tie -> even).
    The fp32 product below is numpy's IEEE multiply, not the oracle's."""
    # midpoint between 1.0 (0x38) and 1.125 (0x39) is 1.0625
    x = np.float32(1.0625) + np.float32(2.0 ** -23)            # 1.0625 + 1ulp
    s = np.float32(1.0) - np.float32(2.0 ** -24)               # just below 1
    exact = Fraction(float(x)) * Fraction(float(s))
    assert exact > Fraction(1.0625)                             # single rounding would give 0x39
    assert np.float32(x * s) == np.float32(1.0625)              # fp32 product is the midpoint
    assert oracle.quantize(np.array([x]), E4M3, s)[0] == 0x38   # tie goes to the even code


@pytest.mark.parametrize("fmt", FMTS)
def test_all_bf16_inputs_scale_one_vs_torch(fmt):
    h = all_bf16_bits()
    q = oracle.quantize(h, fmt, 1.0)
    x = synth.bf16_bits_to_f32(h)
    lib = torch.from_numpy(h.view(np.int16)).view(torch.bfloat16).to(TORCH[fmt]).view(torch.uint8).numpy()
    inside = np.isfinite(x) & (np.abs(x) <= FMAX[fmt])
    assert np.array_equal(q[inside], lib[inside])
    over = np.isfinite(x) & (np.abs(x) > FMAX[fmt])
    assert np.all((q[over] & 0x7F) == MAXCODE[fmt])
    assert np.array_equal(q[over] >> 7, np.signbit(x[over]).astype(np.uint8))
    # the fp32 path sees the same values
    assert np.array_equal(q, oracle.quantize(x, fmt, 1.0))


@pytest.mark.parametrize("fmt,mbits", [(E4M3, 3), (E5M2, 2)])
def test_round_trip_error_bound_on_workload_tensor(fmt, mbits):
    """|decode(q)/s - x| <= 2^-(mbits+1) |x| (1 + 2^-23) wherever the result is normal."""
    h = synth.config2(1 << 18)
    x = synth.bf16_bits_to_f32(h).astype(np.float64)
    a = oracle.amax(h)
    s = oracle.scale_from_amax(a, fmt)
    q = oracle.quantize(h, fmt, s)
    assert (q & 0x7F).max() == MAXCODE[fmt]                      # amax lands on the max code
    back = oracle.dequantize(q, fmt, s)
    min_normal = oracle.decode(fmt, 1 << mbits)
    normal = np.abs(x) * float(s) >= min_normal * (1 + 2.0 ** -20)   # scaled input in the normal range
    err = np.abs(back - x)
    assert np.all(err[normal] <= 2.0 ** -(mbits + 1) * np.abs(x[normal]) * (1 + 2.0 ** -22))
    # below the normal range the error is at most half a subnormal step
    half_step = 0.5 * oracle.decode(fmt, 1) / float(s)
    assert np.all(err[~normal] <= half_step * (1 + 2.0 ** -22))


@pytest.mark.parametrize("fmt", FMTS)
def test_power_of_two_rescaling_of_the_input_changes_nothing(fmt):
    h = synth.config2(1 << 16)
    x = synth.bf16_bits_to_f32(h)
    s = oracle.scale_from_amax(oracle.amax(x), fmt)
    q = oracle.quantize(x, fmt, s)
    for c in (0.125, 64.0):
        xc = (x * np.float32(c)).astype(np.float32)
        sc = oracle.scale_from_amax(oracle.amax(xc), fmt)
        assert sc == s / np.float32(c)
        assert np.array_equal(oracle.quantize(xc, fmt, sc), q)


def test_per_row_helpers_against_numpy_and_the_flat_definitions():
    """amax_rows is numpy's max |x| along axis 1; quantize_rows with equal factors is the flat cast;
    rows are independent (changing one row's factor changes only that row); per-row factors with a
    power-of-two ratio equal a flat cast of the pre-scaled rows (exact multiplication)."""
    x = synth.normal(37 * 53, 9).reshape(37, 53)
    x[5, 7] = -40.0
    assert np.array_equal(oracle.amax_rows(x), np.max(np.abs(x), axis=1))
    h = synth.to_bf16_bits(x.reshape(-1)).reshape(37, 53)
    assert np.array_equal(oracle.amax_rows(h), np.max(np.abs(synth.bf16_bits_to_f32(h)), axis=1))
    for fmt in FMTS:
        s = oracle.scale_from_amax_n(oracle.amax_rows(x), fmt)
        assert all(s[r] == oracle.scale_from_amax(np.max(np.abs(x[r])), fmt) for r in range(37))
        flat = oracle.quantize(x, fmt, 3.0)
        assert np.array_equal(oracle.quantize_rows(x, fmt, np.full(37, 3.0, np.float32)), flat)
        sc = np.full(37, 3.0, np.float32)
        sc[11] = 0.25
        q = oracle.quantize_rows(x, fmt, sc)
        assert np.array_equal(np.delete(q, 11, axis=0), np.delete(flat, 11, axis=0))
        assert np.array_equal(q[11], oracle.quantize(x[11], fmt, 0.25))
        p2 = np.ldexp(1.0, np.arange(37) % 9 - 4).astype(np.float32)
        assert np.array_equal(oracle.quantize_rows(x, fmt, p2), oracle.quantize(x * p2[:, None], fmt, 1.0))
        # the row maximum lands on the largest code of the format, nothing exceeds it
        qs = oracle.quantize_rows(x, fmt, s)
        assert np.all((qs & 0x7F).max(axis=1) == MAXCODE[fmt])
    with pytest.raises(ValueError):
        oracle.quantize_rows(x, E4M3, np.ones(36, np.float32))


def test_scale_from_amax_history():
    for fmt in FMTS:
        h = np.array([0.5, 3.0, 2.0, 0.0], dtype=np.float32)
        assert oracle.scale_from_amax_history(h, fmt) == np.float32(FMAX[fmt] / 3.0)
        assert oracle.scale_from_amax_history(h[:1], fmt) == oracle.scale_from_amax(0.5, fmt)
        assert oracle.scale_from_amax_history(np.zeros(0, np.float32), fmt) == 1.0
        assert oracle.scale_from_amax_history(np.array([1.0, np.nan], np.float32), fmt) == 1.0
        assert oracle.scale_from_amax_history(np.array([1.0, np.inf], np.float32), fmt) == 1.0
