"""Pins for the oracle's encode(): nearest value, ties to even, saturation, specials.

The reference here is the definition itself carried out by other means: exact rational
arithmetic over the list of representable values (pure Python), a dense numpy argmin over
all finite codes, and torch's CPU float8 casts (a library routine that rounds to nearest
even but does not saturate, so it serves below the maximum and for the strict mode).
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import E4M3, E5M2

NFINITE = {E4M3: 127, E5M2: 124}
MAXCODE = {E4M3: 0x7E, E5M2: 0x7B}
TORCH = {E4M3: torch.float8_e4m3fn, E5M2: torch.float8_e5m2}
FMTS = [E4M3, E5M2]


def f32(x):
    return float(np.float32(x))


def next_up(x):
    return float(np.nextafter(np.float32(x), np.float32(np.inf)))


def next_down(x):
    return float(np.nextafter(np.float32(x), np.float32(-np.inf)))


def table(fmt):
    return [oracle.decode(fmt, c) for c in range(NFINITE[fmt])]


def nearest_even_exact(fmt, y, tab):
    """Definition by exhaustive search in exact rationals (saturating)."""
    sign = 0x80 if math.copysign(1.0, y) < 0 else 0
    m = abs(Fraction(y))
    if m >= Fraction(tab[-1]):
        return sign | (len(tab) - 1)
    best, best_d = None, None
    for code, v in enumerate(tab):
        d = abs(m - Fraction(v))
        if best is None or d < best_d or (d == best_d and code % 2 == 0):
            best, best_d = code, d
    return sign | best


@pytest.mark.parametrize("fmt", FMTS)
def test_round_trip_every_finite_code(fmt):
    for b in range(256):
        v = oracle.decode(fmt, b)
        if math.isnan(v):
            continue
        assert oracle.encode(fmt, v) == b, hex(b)
        assert oracle.encode(fmt, v, saturating=False) == b, hex(b)


@pytest.mark.parametrize("fmt", FMTS)
def test_midpoints_go_to_even_and_neighbours_to_nearer(fmt):
    tab = table(fmt)
    for lo in range(len(tab) - 1):
        mid = 0.5 * (tab[lo] + tab[lo + 1])
        assert f32(mid) == mid                      # every midpoint is a float32
        even = lo if lo % 2 == 0 else lo + 1
        assert oracle.encode(fmt, mid) == even, lo
        assert oracle.encode(fmt, -mid) == 0x80 | even, lo
        assert oracle.encode(fmt, next_down(mid)) == lo
        assert oracle.encode(fmt, next_up(mid)) == lo + 1


def _structured_samples(fmt):
    tab = table(fmt)
    ys = [0.0, -0.0]
    for lo in range(len(tab) - 1):
        mid = 0.5 * (tab[lo] + tab[lo + 1])
        for v in (tab[lo], mid, 0.25 * (3 * tab[lo] + tab[lo + 1])):
            ys += [v, next_up(v), next_down(v)] if v > 0 else [v, next_up(v)]
    ys += [tab[-1], next_up(tab[-1]), next_down(tab[-1]), 1e9, 3.0e38,
           float(np.float32(1e-45)), float(np.float32(1e-40)), 2.0 ** -126]
    ys += [-y for y in ys]
    return ys


@pytest.mark.parametrize("fmt", FMTS)
def test_against_exact_rational_search(fmt):
    tab = table(fmt)
    rng = np.random.default_rng(1234 + fmt)
    bits = rng.integers(0, 2 ** 32, size=6000, dtype=np.uint64).astype(np.uint32)
    rnd = [float(v) for v in bits.view(np.float32) if np.isfinite(v)]
    # dense cover of the format's own range, log-uniform
    expo = rng.uniform(-20, 17, size=6000)
    dense = [f32(s * 2.0 ** e) for s, e in zip(rng.choice([-1.0, 1.0], 6000), expo)]
    for y in _structured_samples(fmt) + rnd + dense:
        assert oracle.encode(fmt, y) == nearest_even_exact(fmt, y, tab), (fmt, y.hex())


@pytest.mark.parametrize("fmt", FMTS)
def test_against_dense_argmin(fmt):
    """2 million random float32 inputs against a numpy argmin over every finite code."""
    tab = np.array(table(fmt))
    rng = np.random.default_rng(99 + fmt)
    n = 2_000_000
    # half uniform in bit pattern (all exponents), half log-uniform over the format's range
    bits = rng.integers(0, 2 ** 32, size=n // 2, dtype=np.uint64).astype(np.uint32)
    a = bits.view(np.float32)
    b = (rng.choice([-1.0, 1.0], n // 2) * 2.0 ** rng.uniform(-19, 16.5, n // 2)).astype(np.float32)
    y = np.concatenate([a[np.isfinite(a)], b])
    got = oracle.quantize(y, fmt, 1.0)
    want = np.empty(y.size, dtype=np.uint8)
    for lo in range(0, y.size, 100_000):
        m = np.abs(y[lo:lo + 100_000].astype(np.float64))
        d = np.abs(m[:, None] - tab[None, :])
        dmin = d.min(axis=1, keepdims=True)
        is_min = d == dmin
        # among the (one or two) nearest codes take the even one
        first = np.argmax(is_min, axis=1)
        last = tab.size - 1 - np.argmax(is_min[:, ::-1], axis=1)
        pick = np.where(first % 2 == 0, first, last)
        pick = np.where(m >= tab[-1], tab.size - 1, pick)
        want[lo:lo + 100_000] = pick | (np.signbit(y[lo:lo + 100_000]) << 7)
        assert np.all((last - first <= 1) | (m >= tab[-1]))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("fmt", FMTS)
def test_saturation_and_specials(fmt):
    mx = MAXCODE[fmt]
    vmax = oracle.decode(fmt, mx)
    for y in (vmax, next_up(vmax), vmax * 1.07, vmax * 1.08, 1e9, 3.4e38):
        assert oracle.encode(fmt, y) == mx
        assert oracle.encode(fmt, -y) == 0x80 | mx
    nan = oracle.encode(fmt, float("nan"))
    assert math.isnan(oracle.decode(fmt, nan))
    pinf, ninf = oracle.encode(fmt, math.inf), oracle.encode(fmt, -math.inf)
    if fmt == E4M3:      # no infinities: both become NaN (Section 2, type conversion)
        assert pinf == 0x7F and ninf == 0xFF
    else:                # E5M2 keeps the special value
        assert oracle.decode(fmt, pinf) == math.inf and oracle.decode(fmt, ninf) == -math.inf
        assert (pinf, ninf) == (0x7C, 0xFC)


@pytest.mark.parametrize("fmt", FMTS)
def test_signed_zero_and_underflow(fmt):
    tiny = oracle.decode(fmt, 1)
    assert oracle.encode(fmt, 0.0) == 0x00 and oracle.encode(fmt, -0.0) == 0x80
    assert oracle.encode(fmt, tiny / 2) == 0x00          # tie with zero goes to the even code 0
    assert oracle.encode(fmt, -tiny / 2) == 0x80
    assert oracle.encode(fmt, next_up(tiny / 2)) == 0x01
    assert oracle.encode(fmt, -tiny / 8) == 0x80
    assert oracle.encode(fmt, 1.5 * tiny) == 0x02        # tie between codes 1 and 2
    # seam between the largest subnormal and the smallest normal
    seam_lo = (1 << (3 if fmt == E4M3 else 2)) - 1
    mid = 0.5 * (oracle.decode(fmt, seam_lo) + oracle.decode(fmt, seam_lo + 1))
    assert oracle.encode(fmt, mid) == seam_lo + 1        # seam_lo is odd


@pytest.mark.parametrize("fmt", FMTS)
def test_torch_cast_agrees(fmt):
    """torch's CPU cast: equal to the strict mode everywhere, to the saturating mode
    wherever the input does not exceed the maximum."""
    rng = np.random.default_rng(7 + fmt)
    bits = rng.integers(0, 2 ** 32, size=400_000, dtype=np.uint64).astype(np.uint32)
    y = np.concatenate([
        bits.view(np.float32),
        (rng.choice([-1.0, 1.0], 400_000) * 2.0 ** rng.uniform(-19, 17, 400_000)).astype(np.float32),
        np.array(_structured_samples(fmt), dtype=np.float32),
    ])
    lib = torch.from_numpy(y).to(TORCH[fmt]).view(torch.uint8).numpy()
    strict = oracle.quantize(y, fmt, 1.0, saturating=False)
    sat = oracle.quantize(y, fmt, 1.0, saturating=True)
    vals = oracle.decode_all(fmt)
    nan_in = np.isnan(y)
    assert np.all(np.isnan(vals[lib[nan_in]])) and np.all(np.isnan(vals[strict[nan_in]]))
    lib_nan = np.isnan(vals[lib])
    assert np.array_equal(lib_nan, np.isnan(vals[strict]))      # overflow to NaN in the same places
    ok = ~lib_nan
    assert np.array_equal(lib[ok], strict[ok])
    inside = np.isfinite(y) & (np.abs(y) <= oracle.decode(fmt, MAXCODE[fmt]))
    assert np.array_equal(lib[inside], sat[inside])


def test_nan_codes_are_those_of_the_library_cast():
    """Table 1 gives E5M2 three NaN mantissas and does not say which one a conversion emits; the
    oracle emits S.11111.11 for every NaN input, whatever its payload and sign: the code torch's CPU
    cast (an independent library routine) emits.  E4M3 has a single NaN code per sign."""
    nan_bits = np.array([0x7FC00000, 0xFFC00000, 0x7F800001, 0xFF800001, 0x7FFFFFFF, 0xFFFFFFFF, 0x7FA55AA5], dtype=np.uint32)
    y = nan_bits.view(np.float32)
    for fmt in FMTS:
        lib = torch.from_numpy(y).to(TORCH[fmt]).view(torch.uint8).numpy()
        for sat in (True, False):
            got = oracle.quantize(y, fmt, 1.0, saturating=sat)
            assert np.array_equal(got & 0x7F, np.full(y.size, 0x7F, dtype=np.uint8)), fmt
            assert np.array_equal(got & 0x7F, lib & 0x7F), fmt
    # the sign of a NaN is kept by the oracle (it copies the sign bit like for every other value)
    assert oracle.encode(E5M2, np.float32(np.nan)) in (0x7F, 0xFF)


def test_strict_mode_overflow_points():
    # E4M3: the virtual next grid point is 480; halfway (464) ties to the even code 0x7E
    assert oracle.encode(E4M3, 464.0, saturating=False) == 0x7E
    assert oracle.encode(E4M3, next_up(464.0), saturating=False) == 0x7F
    # E5M2: next grid point 65536; halfway (61440) ties away from the odd code 0x7B -> inf
    assert oracle.encode(E5M2, next_down(61440.0), saturating=False) == 0x7B
    assert oracle.encode(E5M2, 61440.0, saturating=False) == 0x7C
