"""GPU parity, bit for bit, of the scaling-recipe variants of the amax / cast steps against the CPU
oracle: cast + amax in one pass, factor from a history of maxima, per-row amax / factors / cast,
cast + transpose."""
import numpy as np
import pytest
import torch

import oracle
import paper_2209_05433_amd as fp8
from workloads import synth
from gpu_util import to_dev, report_byte_mismatch

pytestmark = pytest.mark.gpu

E4M3, E5M2 = fp8.FP8_E4M3, fp8.FP8_E5M2
FMTS = [E4M3, E5M2]


def tensor(n, seed, dtype, specials=False):
    """Normal values with a few large ones; optionally a sprinkling of NaN / inf / zeros / tiny values."""
    x = synth.normal_with_outliers(n, seed, p=0.001, factor=300.0)
    if specials and n >= 64:
        x[3], x[17], x[n // 2], x[n - 1] = np.nan, np.inf, -np.inf, -0.0
        x[5], x[9] = 1e-30, -3e-41
    return x if dtype == "f32" else synth.to_bf16_bits(x)


def bits_of(x):
    return x.view(np.uint32) if x.dtype == np.float32 else x


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("fmt", FMTS)
def test_quantize_amax_single_pass(fmt, dtype):
    for n, specials in ((1 << 22) + 4096 + 13, False), (100_003, True), (16, False), (5, False), (0, False):
        x = tensor(max(n, 1), 40 + fmt, dtype, specials)[:n]
        dx = to_dev(x) if n else torch.empty(0, dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device="cuda")
        scale = np.float32(37.5)
        q = torch.full((n,), 0xAA, dtype=torch.uint8, device="cuda")
        amax = torch.full((1,), -1.0, device="cuda")
        fp8.fp8_quantize_amax(dx, fmt, to_dev(np.array([scale])), q, amax)
        torch.cuda.synchronize()
        want = oracle.quantize(x, fmt, scale)
        got = q.cpu().numpy()
        assert np.array_equal(got, want), report_byte_mismatch(bits_of(x), got, want)
        a_ref, a = oracle.amax(x), np.float32(amax.item())
        assert (np.isnan(a) and np.isnan(a_ref)) or a == a_ref, (n, a, a_ref)
    # unaligned views take the element-wise path
    x = tensor(70_001, 3, dtype)
    dx = to_dev(x)[1:]
    q = torch.empty(70_001, dtype=torch.uint8, device="cuda")[1:]
    amax = torch.zeros(1, device="cuda")
    fp8.fp8_quantize_amax(dx, fmt, to_dev(np.array([np.float32(2.0)])), q, amax)
    torch.cuda.synchronize()
    assert np.array_equal(q.cpu().numpy(), oracle.quantize(x[1:], fmt, 2.0))
    assert np.float32(amax.item()) == oracle.amax(x[1:])


def test_delayed_scaling_loop_matches_the_oracle():
    """A few steps of the recipe the single-pass cast exists for: the factor of step t comes from the
    maxima of the steps before it; each step casts with it and records its own amax."""
    hist_len, steps, n = 4, 6, 300_000
    hist = torch.zeros(hist_len, device="cuda")
    hist_ref = np.zeros(hist_len, dtype=np.float32)
    scale = torch.zeros(1, device="cuda")
    q = torch.empty(n, dtype=torch.uint8, device="cuda")
    for t in range(steps):
        x = synth.to_bf16_bits(synth.normal(n, 900 + t) * np.float32(1.5 ** t))
        fp8.fp8_scale_from_amax_history(hist, E4M3, scale)
        fp8.fp8_quantize_amax(to_dev(x), E4M3, scale, q, hist[t % hist_len:t % hist_len + 1])
        torch.cuda.synchronize()
        s_ref = oracle.scale_from_amax_history(hist_ref, E4M3)
        assert np.float32(scale.item()) == s_ref, t
        assert np.array_equal(q.cpu().numpy(), oracle.quantize(x, E4M3, s_ref)), t
        hist_ref[t % hist_len] = oracle.amax(x)
        assert np.array_equal(hist.cpu().numpy(), hist_ref), t
    # degenerate histories
    for h in ([], [0.0, 0.0], [1.0, float("nan")], [float("inf")]):
        ht = torch.tensor(h, dtype=torch.float32, device="cuda")
        fp8.fp8_scale_from_amax_history(ht, E5M2, scale)
        assert np.float32(scale.item()) == oracle.scale_from_amax_history(np.array(h, np.float32), E5M2)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_per_row_amax_scale_and_cast(dtype):
    for rows, cols in ((300, 4096), (129, 1000), (7, 33), (1, 1), (64, 16)):
        x = tensor(rows * cols, rows + cols, dtype, specials=cols >= 64).reshape(rows, cols)
        dx = to_dev(x)
        amax = torch.full((rows,), -1.0, device="cuda")
        fp8.fp8_amax_rows(dx, amax)
        torch.cuda.synchronize()
        a_ref = oracle.amax_rows(x)
        assert np.array_equal(amax.cpu().numpy(), a_ref, equal_nan=True), (rows, cols)
        for fmt in FMTS:
            scale = torch.zeros(rows, device="cuda")
            fp8.fp8_scale_from_amax_n(amax, fmt, scale)
            q = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda")
            fp8.fp8_quantize_rows(dx, fmt, scale, q)
            torch.cuda.synchronize()
            s_ref = oracle.scale_from_amax_n(a_ref, fmt)
            assert np.array_equal(scale.cpu().numpy(), s_ref), (rows, cols, fmt)
            want = oracle.quantize_rows(x, fmt, s_ref)
            got = q.cpu().numpy()
            assert np.array_equal(got, want), report_byte_mismatch(bits_of(x).reshape(-1), got.reshape(-1), want.reshape(-1))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("fmt", FMTS)
def test_quantize_transpose(fmt, dtype):
    # (the last two: rows a power of two, where the tiles are walked diagonally, with ragged tiles)
    for rows, cols in ((512, 384), (128, 128), (144, 1040), (16, 16), (33, 20), (1, 7), (300, 128), (4096, 272), (8192, 528)):
        x = tensor(rows * cols, 7 * rows + cols, dtype, specials=rows * cols >= 64).reshape(rows, cols)
        dx = to_dev(x)
        scale = np.float32(11.0)
        want = oracle.quantize(x, fmt, scale)
        for with_q in (True, False):
            q = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda") if with_q else None
            qt = torch.full((cols, rows), 0xAA, dtype=torch.uint8, device="cuda")
            fp8.fp8_quantize_transpose(dx, fmt, to_dev(np.array([scale])), q, qt)
            torch.cuda.synchronize()
            if with_q:
                assert np.array_equal(q.cpu().numpy(), want), (rows, cols, "q")
            got = qt.cpu().numpy()
            assert np.array_equal(got, want.T), "%s: %d bytes of the transposed output differ" % (
                (rows, cols), np.count_nonzero(got != want.T))


def test_quantize_transpose_feeds_the_wgrad_gemm():
    """dW = dY^T X from the transposed bytes equals the transposed-operand GEMM on the plain bytes."""
    rng = np.random.default_rng(12)
    tokens, d_in, d_out = 512, 256, 384
    X = synth.to_bf16_bits(synth.normal(tokens * d_in, 1)).reshape(tokens, d_in)
    dY = synth.to_bf16_bits(synth.normal(tokens * d_out, 2) * np.float32(1e-3)).reshape(tokens, d_out)
    sX = oracle.scale_from_amax(oracle.amax(X), E4M3)
    sY = oracle.scale_from_amax(oracle.amax(dY), E5M2)
    qY = torch.empty((tokens, d_out), dtype=torch.uint8, device="cuda")
    qYt = torch.empty((d_out, tokens), dtype=torch.uint8, device="cuda")
    qX = torch.empty((tokens, d_in), dtype=torch.uint8, device="cuda")
    fp8.fp8_quantize_transpose(to_dev(dY), E5M2, to_dev(np.array([sY])), qY, qYt)
    fp8.fp8_quantize(to_dev(X), E4M3, float(sX), qX)
    dW1 = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    dW2 = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    fp8.fp8_gemm(qYt, E5M2, float(sY), qX, E4M3, float(sX), dW1)
    fp8.fp8_gemm_ex(qY, E5M2, 1, qX, E4M3, 0, dW2, float(sY), float(sX))
    torch.cuda.synchronize()
    S, T = oracle.gemm_rows(oracle.quantize(dY, E5M2, sY).T.copy(), E5M2, oracle.quantize(X, E4M3, sX), E4M3)
    c_ref, bound = oracle.gemm_bound(S, T, sY, sX, oracle.F32)
    for dW in (dW1, dW2):
        assert np.all(np.abs(dW.cpu().numpy().astype(np.float64) - c_ref) <= bound)


def test_config2_size_single_pass_cast():
    """2^28 bf16 elements with outliers (the quantize-only workload), cast + amax in one pass."""
    x = synth.config2()
    dx = to_dev(x)
    n = x.size
    q = torch.empty(n, dtype=torch.uint8, device="cuda")
    amax = torch.zeros(1, device="cuda")
    scale = to_dev(np.array([np.float32(0.1)]))
    fp8.fp8_quantize_amax(dx, E4M3, scale, q, amax)
    torch.cuda.synchronize()
    assert np.float32(amax.item()) == oracle.amax(x)
    want = oracle.quantize(x, E4M3, np.float32(0.1))
    got = q.cpu().numpy()
    assert np.array_equal(got, want), report_byte_mismatch(x, got, want)


def sr_sweep_inputs(fmt):
    """fp32 values over every binade the format sees (normal, subnormal, below the smallest
    subnormal, above the maximum), both signs, with low mantissa bits set, plus grid points,
    midpoints and specials."""
    rng = np.random.default_rng(77 + fmt)
    e = rng.integers(-30, 20, 400_000)
    x = (rng.choice([-1.0, 1.0], e.size) * (1.0 + rng.random(e.size)) * 2.0 ** e).astype(np.float32)
    vals = oracle.decode_all(fmt)
    finite = vals[np.isfinite(vals)].astype(np.float32)
    mids = ((finite[:-1].astype(np.float64) + finite[1:]) / 2).astype(np.float32)
    extra = np.array([0.0, -0.0, np.nan, np.inf, -np.inf, 1e-45, -1e-45, 3e38, -3e38], dtype=np.float32)
    bits = rng.integers(0, 2 ** 32, 100_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    return np.concatenate([x, finite, mids, np.nextafter(mids, np.float32(0)), extra, bits])


@pytest.mark.parametrize("fmt", FMTS)
def test_stochastic_rounding_cast(fmt):
    x = sr_sweep_inputs(fmt)
    n = x.size
    for seed in (0, 0xDEADBEEFCAFEF00D):
        q = torch.full((n,), 0xAA, dtype=torch.uint8, device="cuda")
        fp8.fp8_quantize_sr(to_dev(x), fmt, 1.0, seed, q)
        torch.cuda.synchronize()
        want = oracle.quantize_sr(x, fmt, 1.0, seed)
        got = q.cpu().numpy()
        nan_in = np.isnan(x)
        assert np.array_equal(got[~nan_in], want[~nan_in]), report_byte_mismatch(x.view(np.uint32)[~nan_in], got[~nan_in], want[~nan_in])
        assert np.all((got[nan_in] & 0x7F) == (0x7F if fmt == E4M3 else 0x7F))
    # bf16 input, device scale, a scale that is not a power of two; unaligned view (element path)
    h = tensor(300_007, 5, "bf16", specials=True)
    s = np.float32(13.7)
    q = torch.empty(h.size, dtype=torch.uint8, device="cuda")
    fp8.fp8_quantize_sr(to_dev(h), fmt, to_dev(np.array([s])), 99, q)
    torch.cuda.synchronize()
    assert np.array_equal(q.cpu().numpy(), oracle.quantize_sr(h, fmt, s, 99))
    q2 = torch.empty(h.size, dtype=torch.uint8, device="cuda")[3:]
    fp8.fp8_quantize_sr(to_dev(h)[3:], fmt, float(s), 99, q2)
    torch.cuda.synchronize()
    assert np.array_equal(q2.cpu().numpy(), oracle.quantize_sr(h[3:], fmt, s, 99))


@pytest.mark.parametrize("fmt", FMTS)
def test_stochastic_rounding_carry_boundaries_and_a_large_sweep(fmt):
    """The kernel rounds through the converter instructions; the oracle through the definition.
    (1) Inputs built, element by element, from the element's own random bits r so that T + r is
    exactly 2^16 - 1 (must stay) or 2^16 (must go up), with every bit below T set: normal and
    subnormal results.  (2) 2^24 random fp32 patterns."""
    seed = 0x1234ABCD5678
    mb = 3 if fmt == E4M3 else 2
    drop = 23 - mb
    n = 40_000
    rng = np.random.default_rng(5 + fmt)
    r = np.array([oracle.sr_bits(seed, i) for i in range(n)], dtype=np.int64)
    T = np.where(np.arange(n) % 2 == 0, 65535 - r, (65536 - r) & 0xFFFF)
    low = (1 << (drop - 16)) - 1
    # normal results: random exponent inside the format's normal range, random kept mantissa
    emin, emax = (-6, 7) if fmt == E4M3 else (-14, 14)
    e = rng.integers(emin, emax + 1, n)
    kept = rng.integers(0, 1 << mb, n)
    bits = ((rng.integers(0, 2, n) << 31) | ((e + 127) << 23) | (kept << drop) | (T << (drop - 16)) | low).astype(np.uint32)
    x = bits.view(np.float32).copy()
    # subnormal results (every fourth element): |y| = (k 2^16 + T + (1 - 2^-4)) 2^-16 steps
    step_log2 = (1 - (7 if fmt == E4M3 else 15)) - mb
    sub = np.arange(n) % 4 >= 2
    k = rng.integers(0, 1 << mb, n)
    mag = ((k * 65536 + T) * 16 + 15).astype(np.float64) * 2.0 ** (step_log2 - 20)
    x[sub] = (np.where(rng.integers(0, 2, n) == 1, -1.0, 1.0) * mag).astype(np.float32)[sub]
    assert np.array_equal(x[sub].astype(np.float64), (np.sign(x[sub]) * mag[sub]))            # exactly representable
    q = torch.empty(n, dtype=torch.uint8, device="cuda")
    fp8.fp8_quantize_sr(to_dev(x), fmt, 1.0, seed, q)
    torch.cuda.synchronize()
    want = oracle.quantize_sr(x, fmt, 1.0, seed)
    got = q.cpu().numpy()
    assert np.array_equal(got, want), report_byte_mismatch(x.view(np.uint32), got, want)
    # the construction does what it says: odd elements sit one code above the truncation, even ones on it
    head = 2000
    truncated = np.array([oracle.encode_sr(fmt, v, 0) for v in x[:head]], dtype=np.uint8)     # r = 0 never goes up
    stays = want[:head] == truncated
    assert stays[0::2].all() and not stays[1::2][r[1:head:2] > 0].any()

    m = 1 << 24
    big = rng.integers(0, 2 ** 32, m, dtype=np.uint64).astype(np.uint32).view(np.float32)
    q = torch.empty(m, dtype=torch.uint8, device="cuda")
    fp8.fp8_quantize_sr(to_dev(big), fmt, 1.0, seed + 1, q)
    torch.cuda.synchronize()
    want = oracle.quantize_sr(big, fmt, 1.0, seed + 1)
    got = q.cpu().numpy()
    ok = ~np.isnan(big)
    assert np.array_equal(got[ok], want[ok]), report_byte_mismatch(big.view(np.uint32)[ok], got[ok], want[ok])
    assert np.all((got[~ok] & 0x7F) == 0x7F)


def test_stochastic_rounding_is_unbiased_on_the_device():
    n = 1 << 22
    x = torch.full((n,), 0.3, device="cuda")
    q = torch.empty(n, dtype=torch.uint8, device="cuda")
    fp8.fp8_quantize_sr(x, E4M3, 3.7, 1234, q)
    mean = fp8_mean(q, E4M3)
    y = float(np.float32(0.3) * np.float32(3.7))
    assert abs(mean - y) < 1e-3 * y          # RNE would be off by 1.2 % here (1.11 -> 1.125)


def fp8_mean(q, fmt):
    out = torch.empty(q.numel(), dtype=torch.float32, device="cuda")
    fp8.fp8_dequantize(q, fmt, 1.0, out)
    torch.cuda.synchronize()
    return float(out.double().mean().item())
