"""Pins for the oracle's stochastic rounding and its counter-based generator."""
import numpy as np
import pytest

import oracle
from oracle import E4M3, E5M2

FMTS = [E4M3, E5M2]
MAXCODE = {E4M3: 0x7E, E5M2: 0x7B}


def test_philox_known_answers():
    """Known-answer vectors of Philox4x32-10 published with the generator (Random123 kat_vectors)."""
    kat = [
        ([0, 0, 0, 0], [0, 0], [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]),
        ([0xffffffff] * 4, [0xffffffff] * 2, [0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd]),
        ([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], [0xa4093822, 0x299f31d0],
         [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]),
    ]
    for ctr, key, want in kat:
        assert [int(v) for v in oracle.philox4x32(ctr, key)] == want


def test_sr_bits_field_order():
    seed = 0x0123456789ABCDEF
    w = oracle.philox4x32([5, 0, 0, 0], [seed & 0xffffffff, seed >> 32])
    fields = [oracle.sr_bits(seed, 40 + f) for f in range(8)]
    assert fields == [int(w[f // 2] >> (16 * (f % 2))) & 0xFFFF for f in range(8)]
    # a block index above 2^32 reaches the second counter word
    w = oracle.philox4x32([1, 3, 0, 0], [7, 0])
    assert oracle.sr_bits(7, ((3 << 32) + 1) * 8) == int(w[0]) & 0xFFFF


@pytest.mark.parametrize("fmt", FMTS)
def test_probability_of_rounding_up_is_the_position_between_the_neighbours(fmt):
    """Over all 2^16 values of r exactly floor(t * 2^16) of them round up: checked by brute force
    for values in the normal range, in the subnormal range, next to zero and next to the maximum."""
    vals = oracle.decode_all(fmt)
    rng = np.random.default_rng(3 + fmt)
    for code in [0, 1, 2, (9 if fmt == E4M3 else 5), 0x30, 0x55, MAXCODE[fmt] - 1]:
        lo, hi = vals[code], vals[code + 1]
        for frac in (0.0, 1.0 / 65536, 0.25, 0.5, 0.75 + 1.0 / 1024, 1 - 1.0 / 65536, float(rng.random())):
            y = np.float32(lo + frac * (hi - lo))
            t = (float(y) - lo) / (hi - lo)
            ups = sum(oracle.encode_sr(fmt, y, r) == code + 1 for r in range(65536))
            downs = sum(oracle.encode_sr(fmt, -y, r) == (0x80 | code) for r in range(0, 65536, 257))
            if float(y) == hi:                       # rounded onto the next grid point by the fp32 cast
                continue
            assert ups == int(np.floor(t * 65536)), (fmt, code, frac)
            assert downs > 0 or t * 65536 >= 65535


@pytest.mark.parametrize("fmt", FMTS)
def test_grid_points_never_move_and_extremes(fmt):
    vals = oracle.decode_all(fmt)
    for code in range(MAXCODE[fmt] + 1):
        for r in (0, 1, 0x8000, 0xFFFF):
            assert oracle.encode_sr(fmt, np.float32(vals[code]), r) == code
            assert oracle.encode_sr(fmt, np.float32(-vals[code]), r) == (0x80 | code)
    # r = 0 truncates toward zero; r = 0xFFFF rounds every off-grid value with T >= 1 away from zero
    rng = np.random.default_rng(8)
    y = (rng.standard_normal(5000) * 2.0 ** rng.integers(-12, 8, 5000)).astype(np.float32)
    y = y[np.abs(y) < vals[MAXCODE[fmt]]]
    down = np.array([oracle.encode_sr(fmt, v, 0) for v in y])
    assert np.all(np.abs(vals[down]) <= np.abs(y)) and np.all(np.signbit(vals[down]) == np.signbit(y))
    rne = oracle.quantize(y, fmt, 1.0)
    assert np.all(np.abs((down & 0x7F).astype(int) - (rne & 0x7F).astype(int)) <= 1)
    # saturation and specials as in the deterministic cast
    big = np.float32(vals[MAXCODE[fmt]] * 4)
    assert oracle.encode_sr(fmt, big, 0xFFFF) == MAXCODE[fmt] and oracle.encode_sr(fmt, -big, 0) == 0x80 | MAXCODE[fmt]
    assert oracle.encode_sr(fmt, np.float32(np.nan), 5) == oracle.encode(fmt, np.float32(np.nan))
    assert oracle.encode_sr(fmt, np.float32(-np.inf), 5) == oracle.encode(fmt, np.float32(-np.inf))


@pytest.mark.parametrize("fmt", FMTS)
def test_quantize_sr_is_unbiased_and_reproducible(fmt):
    n = 200_000
    x = np.full(n, 0.3, dtype=np.float32)
    scale = np.float32(3.7)
    q1 = oracle.quantize_sr(x, fmt, scale, seed=11)
    q2 = oracle.quantize_sr(x, fmt, scale, seed=11)
    q3 = oracle.quantize_sr(x, fmt, scale, seed=12)
    assert np.array_equal(q1, q2) and not np.array_equal(q1, q3)
    vals = oracle.decode_all(fmt)
    y = float(np.float32(x[0] * scale))
    assert set(np.unique(q1)) == {oracle.encode_sr(fmt, np.float32(y), 0), oracle.encode_sr(fmt, np.float32(y), 0) + 1}
    step = vals[q1.max()] - vals[q1.min()]
    assert abs(vals[q1].mean() - y) < 4 * step / np.sqrt(n) + step * 2.0 ** -16
    # element i uses sr_bits(seed, i)
    for i in (0, 7, 8, 12345):
        assert q1[i] == oracle.encode_sr(fmt, np.float32(y), oracle.sr_bits(11, i))
