"""Pins for the oracle's decode(): what the paper prints and what IEEE/library routines fix.

Every check here compares the oracle with something that is not the oracle: Table 1 rows
(tests/golden/table1_formats.txt), the facts of Section 3.1 (tests/golden/section31_facts.txt),
numpy's float16 and torch's float8 dtypes (library decoders), and closed forms.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import E4M3, E5M2

FMT = {"E4M3": E4M3, "E5M2": E5M2}


def _rows(path):
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [c.strip() for c in line.split("|")]


def _pattern_to_bytes(pattern):
    """'S.1111.110' -> (0x7E, 0xFE)"""
    s, e, m = pattern.split(".")
    assert s == "S"
    mag = int(e + m, 2)
    assert len(e + m) == 7
    return mag, mag | 0x80


def test_table1_rows(golden_dir):
    n = 0
    for fmt, pattern, kind, mant, power, decimal, _where in _rows(
            os.path.join(golden_dir, "table1_formats.txt")):
        pos, neg = _pattern_to_bytes(pattern)
        vp, vn = oracle.decode(FMT[fmt], pos), oracle.decode(FMT[fmt], neg)
        if kind == "nan":
            assert math.isnan(vp) and math.isnan(vn)
        elif kind == "inf":
            assert vp == math.inf and vn == -math.inf
        elif kind == "zero":
            assert vp == 0.0 and vn == 0.0
            assert math.copysign(1.0, vp) == 1.0 and math.copysign(1.0, vn) == -1.0
        else:
            want = float(mant) * 2.0 ** int(power)
            assert vp == want and vn == -want, (fmt, pattern)
            if decimal != "-":
                assert vp == float(decimal)
        n += 1
    assert n == 15


def _facts(golden_dir):
    return {k: v.split() for k, v, _ in _rows(os.path.join(golden_dir, "section31_facts.txt"))}


def test_section31_e4m3_extension(golden_dir):
    facts = _facts(golden_dir)
    vals = oracle.decode_all(E4M3)
    # the seven magnitudes at biased exponent 1111 are codes 0x78..0x7E
    got = [vals[0x78 + i] for i in range(7)]
    assert got == [float(x) for x in facts["e4m3_magnitudes_at_exponent_1111"]]
    # largest value below that exponent
    assert vals[0x77] == float(facts["e4m3_max_without_extension"][0])
    finite = vals[np.isfinite(vals)]
    assert float(facts["e4m3_not_representable"][0]) not in set(np.abs(finite))
    assert np.isinf(vals).sum() == int(facts["e4m3_infinities"][0])


def _binades(values):
    pos = values[np.isfinite(values) & (values > 0)]
    return len({math.floor(math.log2(v)) for v in pos})


def test_section31_binade_counts(golden_dir):
    facts = _facts(golden_dir)
    v4 = oracle.decode_all(E4M3)
    v5 = oracle.decode_all(E5M2)
    assert _binades(v4) == int(facts["e4m3_binades"][0])
    assert _binades(v4[:0x78]) == int(facts["e4m3_binades_without_extension"][0])
    assert _binades(v5) == int(facts["e5m2_binades_with_subnormals"][0])


def test_pattern_census():
    v4 = oracle.decode_all(E4M3)
    assert np.isnan(v4).sum() == 2 and np.isinf(v4).sum() == 0
    assert (v4 == 0).sum() == 2
    assert len(set(v4[np.isfinite(v4) & (v4 > 0)])) == 126
    assert set(np.flatnonzero(np.isnan(v4))) == {0x7F, 0xFF}
    v5 = oracle.decode_all(E5M2)
    assert np.isnan(v5).sum() == 6 and np.isinf(v5).sum() == 2
    assert (v5 == 0).sum() == 2
    assert len(set(v5[np.isfinite(v5) & (v5 > 0)])) == 123
    assert set(np.flatnonzero(np.isinf(v5))) == {0x7C, 0xFC}


@pytest.mark.parametrize("fmt,nfinite", [(E4M3, 127), (E5M2, 124)])
def test_integer_order_is_magnitude_order(fmt, nfinite):
    """Same-sign patterns sort as integers (Section 3.1: comparison with integer operations)."""
    v = oracle.decode_all(fmt)
    mags = v[:nfinite]
    assert np.all(np.diff(mags) > 0)
    assert np.array_equal(v[0x80:0x80 + nfinite], -mags)


def test_e5m2_is_truncated_float16():
    """Section 3: E5M2 is IEEE half precision with fewer mantissa bits."""
    codes = np.arange(256, dtype=np.uint16)
    half = (codes << 8).view(np.float16).astype(np.float64)
    got = oracle.decode_all(E5M2)
    assert np.array_equal(np.isnan(half), np.isnan(got))
    ok = ~np.isnan(half)
    assert np.array_equal(half[ok], got[ok])
    assert np.array_equal(np.signbit(half[ok]), np.signbit(got[ok]))


@pytest.mark.parametrize("fmt,tdtype", [(E4M3, torch.float8_e4m3fn), (E5M2, torch.float8_e5m2)])
def test_decode_matches_torch_float8(fmt, tdtype):
    """Library cross-check: torch's float8 dtypes decode the same 256 patterns."""
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    lib = codes.view(tdtype).to(torch.float64).numpy()
    got = oracle.decode_all(fmt)
    assert np.array_equal(np.isnan(lib), np.isnan(got))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], got[ok])


@pytest.mark.parametrize("fmt,mbits,bias,nfinite", [(E4M3, 3, 7, 127), (E5M2, 2, 15, 124)])
def test_spacing_closed_form(fmt, mbits, bias, nfinite):
    """Inside binade e the step is 2^(e-mbits); subnormals step by 2^(1-bias-mbits)."""
    v = oracle.decode_all(fmt)[:nfinite]
    for code in range(nfinite - 1):
        E = code >> mbits
        e = (E if E > 0 else 1) - bias
        assert v[code + 1] - v[code] == 2.0 ** (e - mbits), code
    assert v[1] == 2.0 ** (1 - bias - mbits)
