"""GPU parity: fp8_amax, fp8_scale_from_amax, fp8_quantize(+_dscale) against the CPU oracle.
Everything is compared bit for bit.  Both implementations of the rounding step (integer
bit manipulation and the hardware converter) are checked."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2209_05433_amd as fp8
from workloads import synth
from gpu_util import to_dev, cast_path, report_byte_mismatch

pytestmark = pytest.mark.gpu

FMTS = [fp8.FP8_E4M3, fp8.FP8_E5M2]
PATHS = ["bits", "cvt"]


def gpu_quantize(x_np, fmt, scale, path="bits"):
    x = to_dev(x_np)
    q = torch.empty(x.numel(), dtype=torch.uint8, device="cuda")
    with cast_path(path):
        fp8.fp8_quantize(x, fmt, float(scale), q)
    torch.cuda.synchronize()
    return q.cpu().numpy()


def gpu_amax(x_np):
    x = to_dev(x_np)
    out = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    fp8.fp8_amax(x, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()[0]


def structured_fp32_patterns():
    """Every sign/exponent/top-12-mantissa-bit combination with four low-bit fillers:
    covers each rounding position of both formats with zero and non-zero sticky bits."""
    hi = np.arange(1 << 21, dtype=np.uint32) << 11
    return np.concatenate([hi | lo for lo in (0x000, 0x001, 0x400, 0x7FF)]).astype(np.uint32)


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("fmt", FMTS)
def test_quantize_structured_fp32_sweep(fmt, path):
    bits = structured_fp32_patterns()
    x = bits.view(np.float32)
    got = gpu_quantize(x, fmt, 1.0, path)
    want = oracle.quantize(x, fmt, 1.0)
    assert np.array_equal(got, want), report_byte_mismatch(bits, got, want)


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("fmt", FMTS)
def test_quantize_all_bf16_inputs_several_scales(fmt, path):
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    h = np.tile(h, 4)[: 4 * 65536 - 5]            # a ragged tail for the vector kernel
    for scale in (1.0, 0.0973, 448.0 / 4657.0, 57344.0 / 3.1e-4, 2.0 ** -20, 3.0e38, 1e-30, -1.5):
        got = gpu_quantize(h, fmt, scale, path)
        want = oracle.quantize(h, fmt, np.float32(scale))
        assert np.array_equal(got, want), "scale %g\n%s" % (scale, report_byte_mismatch(h, got, want))


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("fmt", FMTS)
def test_quantize_random_fp32_with_real_scales(fmt, path):
    rng = np.random.default_rng(77 + fmt)
    x = (rng.standard_normal(3_000_017) * 2.0 ** rng.integers(-12, 12, 3_000_017)).astype(np.float32)
    x[::1000] = [np.inf, -np.inf, np.nan, 0.0, -0.0][fmt % 5]
    x[5::1777] = np.nan
    x[7::1999] = -np.inf
    for scale in (0.3717, 1234.5, 7.7e-3):
        got = gpu_quantize(x, fmt, scale, path)
        want = oracle.quantize(x, fmt, np.float32(scale))
        assert np.array_equal(got, want), report_byte_mismatch(x.view(np.uint32), got, want)


@pytest.mark.parametrize("fmt", FMTS)
def test_quantize_edge_sizes_and_alignment(fmt):
    rng = np.random.default_rng(5)
    base = rng.standard_normal(5000).astype(np.float32) * 30
    hb = synth.to_bf16_bits(base)
    for n in (0, 1, 15, 16, 17, 255, 256, 257, 4099):
        for arr in (base[:n], hb[:n]):
            got = gpu_quantize(arr, fmt, 2.5, "cvt")
            assert np.array_equal(got, oracle.quantize(arr, fmt, np.float32(2.5))), n
    # misaligned views of device buffers (element-aligned only): scalar kernels
    for arr, off in ((base, 1), (hb, 3)):
        x = to_dev(arr)[off:off + 1001]
        qbuf = torch.zeros(2048, dtype=torch.uint8, device="cuda")
        q = qbuf[5:5 + 1001]
        fp8.fp8_quantize(x, fmt, 0.75, q)
        a = torch.zeros(1, device="cuda")
        fp8.fp8_amax(x, a)
        torch.cuda.synchronize()
        assert np.array_equal(q.cpu().numpy(), oracle.quantize(arr[off:off + 1001], fmt, np.float32(0.75)))
        assert qbuf[:5].sum().item() == 0 and qbuf[5 + 1001:].sum().item() == 0     # nothing outside
        assert a.item() == oracle.amax(arr[off:off + 1001])


def test_amax_matches_oracle():
    rng = np.random.default_rng(9)
    for n in (0, 1, 7, 8, 9, 1023, 1 << 20, (1 << 22) + 13):
        x = (rng.standard_normal(n) * 2.0 ** rng.integers(-8, 8, n)).astype(np.float32)
        assert gpu_amax(x) == oracle.amax(x), n
        h = synth.to_bf16_bits(x)
        assert gpu_amax(h) == oracle.amax(h), n
    # the maximum in the very last (tail) element and in the very first
    x = np.ones(100_003, dtype=np.float32)
    x[-1] = -77.0
    assert gpu_amax(x) == 77.0 and gpu_amax(synth.to_bf16_bits(x)) == 77.0
    x[-1] = 1.0
    x[0] = -99.0
    assert gpu_amax(x) == 99.0
    assert gpu_amax(np.array([-0.0], dtype=np.float32)) == 0.0


def test_amax_specials():
    x = np.ones(70_000, dtype=np.float32)
    x[12345] = -np.inf
    assert gpu_amax(x) == np.inf and gpu_amax(synth.to_bf16_bits(x)) == np.inf
    x[54321] = np.nan
    assert np.isnan(gpu_amax(x)) and np.isnan(gpu_amax(synth.to_bf16_bits(x)))
    assert np.isnan(oracle.amax(x))


@pytest.mark.parametrize("fmt", FMTS)
def test_device_scale_pipeline_without_host_round_trip(fmt):
    """amax -> scale -> cast entirely on the stream, compared with the oracle's three steps."""
    h = synth.config2(1 << 22)
    x = to_dev(h)
    amax = torch.zeros(1, device="cuda")
    scale = torch.zeros(1, device="cuda")
    q = torch.empty(h.size, dtype=torch.uint8, device="cuda")
    with cast_path("cvt"):
        fp8.fp8_amax(x, amax)
        fp8.fp8_scale_from_amax(amax, fmt, scale)
        fp8.fp8_quantize_dscale(x, fmt, scale, q)
    torch.cuda.synchronize()
    a = oracle.amax(h)
    s = oracle.scale_from_amax(a, fmt)
    assert amax.item() == a and np.float32(scale.item()) == s
    want = oracle.quantize(h, fmt, s)
    got = q.cpu().numpy()
    assert np.array_equal(got, want), report_byte_mismatch(h, got, want)
    assert (got & 0x7F).max() == (0x7E if fmt == fp8.FP8_E4M3 else 0x7B)


@pytest.mark.parametrize("fmt", FMTS)
def test_amax_scale_in_one_launch_equals_the_oracle_and_reuses_its_workspace(fmt):
    """fp8_amax_scale: amax and scale out of one launch, no cell cleared beforehand.  One workspace is
    used for a sequence of calls of very different sizes (1024 workgroups, then 1, then a few): a
    partial maximum left over from a larger call must not enter a smaller one, and the ticket must
    come back to zero every time.  Also NaN / inf / empty / unaligned inputs, and amax alone."""
    rng = np.random.default_rng(19)
    ws = torch.zeros(fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
    NCOUNTER = 32 * 33                                  # the counters' part of the workspace; partial maxima follow
    ws[NCOUNTER:] = 0x7F000000                          # stale partials (a huge magnitude) must never be read
    amax = torch.full((1,), -1.0, device="cuda")
    scale = torch.full((1,), -1.0, device="cuda")
    sizes = [(1 << 24) + 5, 3, 1 << 20, 0, 70_001, 1 << 24, 9]
    for k, n in enumerate(sizes):
        x = (rng.standard_normal(n) * np.float32(2.0 ** (8 - 3 * k))).astype(np.float32)     # later calls hold smaller values
        for h in (x, synth.to_bf16_bits(x)):
            d = to_dev(h) if n else torch.empty(0, dtype=torch.float32 if h.dtype == np.float32 else torch.bfloat16, device="cuda")
            fp8.fp8_amax_scale(d, fmt, amax, scale, ws)
            torch.cuda.synchronize()
            a = oracle.amax(h)
            assert amax.item() == a, (n, h.dtype)
            assert np.float32(scale.item()) == oracle.scale_from_amax(a, fmt), (n, h.dtype)
            assert int(ws[:NCOUNTER].abs().sum().item()) == 0, "a counter was left non-zero"
    x = np.ones(300_000, dtype=np.float32)
    x[123_456] = -np.inf
    fp8.fp8_amax_scale(to_dev(x), fmt, amax, scale, ws)
    assert amax.item() == np.inf and scale.item() == 1.0
    x[7] = np.nan
    fp8.fp8_amax_scale(to_dev(synth.to_bf16_bits(x)), fmt, amax, scale, ws)
    assert np.isnan(amax.item()) and scale.item() == 1.0
    # unaligned input (element path) and amax without a scale
    buf = to_dev(np.arange(10_000, dtype=np.float32) - 5000.0)
    scale.fill_(-3.0)
    fp8.fp8_amax_scale(buf[1:9_998], fmt, amax, None, ws)
    torch.cuda.synchronize()
    assert amax.item() == 4999.0 and scale.item() == -3.0 and int(ws[:NCOUNTER].abs().sum().item()) == 0
    # the pipeline with the one-launch form, bit for bit
    h = synth.config2(1 << 22)
    xd = to_dev(h)
    q = torch.empty(h.size, dtype=torch.uint8, device="cuda")
    fp8.fp8_amax_scale(xd, fmt, amax, scale, ws)
    fp8.fp8_quantize_dscale(xd, fmt, scale, q)
    torch.cuda.synchronize()
    s_ref = oracle.scale_from_amax(oracle.amax(h), fmt)
    assert np.float32(scale.item()) == s_ref
    assert np.array_equal(q.cpu().numpy(), oracle.quantize(h, fmt, s_ref))


def test_device_scale_rule_degenerate_cases():
    for a in (0.0, np.inf, np.nan, 1e-45, 3.0, 4567.0):
        for fmt in FMTS:
            amax = torch.tensor([a], dtype=torch.float32, device="cuda")
            scale = torch.zeros(1, device="cuda")
            fp8.fp8_scale_from_amax(amax, fmt, scale)
            assert np.float32(scale.item()) == oracle.scale_from_amax(np.float32(a), fmt), a


@pytest.mark.parametrize("fmt", FMTS)
def test_hardware_converter_equals_bit_path_on_all_fp32_patterns(fmt):
    """All 2^32 single-precision inputs: the two implementations of the rounding step give
    the same bytes (compared on the device); with the structured sweep above pinning the
    bit path to the oracle this extends the pin to every input."""
    chunk = 1 << 27
    q1 = torch.empty(chunk, dtype=torch.uint8, device="cuda")
    q2 = torch.empty(chunk, dtype=torch.uint8, device="cuda")
    base = torch.arange(chunk, dtype=torch.int64, device="cuda")
    for c in range((1 << 32) // chunk):
        bits = (base + c * chunk)
        x = torch.where(bits >= (1 << 31), bits - (1 << 32), bits).to(torch.int32).view(torch.float32)
        with cast_path("bits"):
            fp8.fp8_quantize(x, fmt, 1.0, q1)
        with cast_path("cvt"):
            fp8.fp8_quantize(x, fmt, 1.0, q2)
        if not torch.equal(q1, q2):
            bad = torch.nonzero(q1 != q2).flatten()[:8].cpu().numpy()
            xb = x.view(torch.int32).cpu().numpy().view(np.uint32)
            a, b = q1.cpu().numpy(), q2.cpu().numpy()
            raise AssertionError("chunk %d: " % c + ", ".join(
                "0x%08x bits->0x%02x cvt->0x%02x" % (xb[i], a[i], b[i]) for i in bad))


@pytest.mark.skipif(bool(os.environ.get("FP8MM_SKIP_FULL_SWEEP")), reason="FP8MM_SKIP_FULL_SWEEP is set")
@pytest.mark.parametrize("fmt", FMTS)
def test_full_fp32_sweep_against_oracle(fmt):
    """Every one of the 2^32 fp32 bit patterns through the cast (integer rounding path; the converter
    path is compared with it on the same 2^32 inputs above) against the oracle: about 20 s per format
    with 16 host cores."""
    chunk = 1 << 26
    for c in range((1 << 32) // chunk):
        bits = (np.arange(chunk, dtype=np.uint64) + c * chunk).astype(np.uint32)
        x = bits.view(np.float32)
        got = gpu_quantize(x, fmt, 1.0, "bits")
        want = oracle.quantize(x, fmt, 1.0)
        assert np.array_equal(got, want), report_byte_mismatch(bits, got, want)
        print("chunk %d/64 ok" % c, flush=True)


# ---- conversion variants: strict (non-saturating) cast and the way back ---------------------------

@pytest.mark.parametrize("fmt", FMTS)
def test_strict_cast_matches_oracle(fmt):
    bits = structured_fp32_patterns()
    x = bits.view(np.float32)
    xd = to_dev(x)
    q = torch.empty(x.size, dtype=torch.uint8, device="cuda")
    fp8.fp8_quantize_ex(xd, fmt, 1.0, fp8.FP8_QUANT_NOSAT, q)
    torch.cuda.synchronize()
    want = oracle.quantize(x, fmt, 1.0, saturating=False)
    got = q.cpu().numpy()
    assert np.array_equal(got, want), report_byte_mismatch(bits, got, want)
    # bf16 input, real scale from device memory, ragged and misaligned
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)[:65536 - 3]
    s = torch.tensor([3.3], dtype=torch.float32, device="cuda")
    hd = to_dev(h)
    q = torch.empty(h.size + 1, dtype=torch.uint8, device="cuda")
    fp8.fp8_quantize_ex(hd, fmt, s, fp8.FP8_QUANT_NOSAT, q[1:])
    torch.cuda.synchronize()
    assert np.array_equal(q[1:].cpu().numpy(), oracle.quantize(h, fmt, np.float32(3.3), saturating=False))
    # flags = 0 is the saturating cast
    fp8.fp8_quantize_ex(hd, fmt, 3.3, 0, q[1:])
    torch.cuda.synchronize()
    assert np.array_equal(q[1:].cpu().numpy(), oracle.quantize(h, fmt, np.float32(3.3)))
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_quantize_ex(hd, fmt, 1.0, 8, q[1:])


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("fmt", FMTS)
def test_dequantize_matches_oracle(fmt, out_dtype):
    rng = np.random.default_rng(4)
    q_np = np.concatenate([np.arange(256, dtype=np.uint8), rng.integers(0, 256, 100_003).astype(np.uint8)])
    for scale in (1.0, 0.0973, 448.0 / 4657.0, 1234.5):
        qd = to_dev(q_np)
        out = torch.empty(q_np.size, dtype=out_dtype, device="cuda")
        fp8.fp8_dequantize(qd, fmt, scale, out)
        torch.cuda.synchronize()
        exact = oracle.dequantize(q_np, fmt, np.float32(scale))            # decode / scale in fp64
        got = out.float().cpu().numpy().astype(np.float64)
        nan = np.isnan(exact)
        assert np.array_equal(np.isnan(got), nan)
        inf = np.isinf(exact)
        assert np.array_equal(got[inf], exact[inf])
        ok = ~nan & ~inf
        # correctly rounded single-precision quotient (numpy's IEEE division), then bf16 RNE if asked
        want32 = (oracle.decode_all(fmt)[q_np].astype(np.float32) / np.float32(scale))
        if out_dtype == torch.float32:
            assert np.array_equal(got[ok], want32[ok].astype(np.float64))
            assert np.all(np.abs(got[ok] - exact[ok]) <= 0.5 * oracle.ulp(exact[ok], oracle.F32) * (1 + 1e-9))
        else:
            want16 = torch.from_numpy(want32).to(torch.bfloat16).float().numpy().astype(np.float64)
            assert np.array_equal(got[ok], want16[ok])
            assert np.all(np.abs(got[ok] - exact[ok]) <= 0.5 * oracle.ulp(exact[ok], oracle.BF16) * (1 + 2.0 ** -15))
        assert np.array_equal(np.signbit(got[ok]), np.signbit(exact[ok]))


@pytest.mark.parametrize("fmt", FMTS)
def test_cast_and_back_is_the_simulated_fp8_of_the_paper(fmt):
    """Cast to FP8 and back to the 16-bit type (how the paper's experiments simulate FP8,
    Section 4): the round trip is idempotent and stays within half an FP8 step."""
    h = synth.config2(1 << 20)
    x = to_dev(h)
    amax = torch.zeros(1, device="cuda"); scale = torch.zeros(1, device="cuda")
    q = torch.empty(h.size, dtype=torch.uint8, device="cuda")
    back = torch.empty(h.size, dtype=torch.float32, device="cuda")
    q2 = torch.empty_like(q)
    fp8.fp8_amax(x, amax)
    fp8.fp8_scale_from_amax(amax, fmt, scale)
    fp8.fp8_quantize_dscale(x, fmt, scale, q)
    fp8.fp8_dequantize(q, fmt, scale, back)
    fp8.fp8_quantize_dscale(back, fmt, scale, q2)
    torch.cuda.synchronize()
    same = (q == q2)
    # a value can move by one code only if decode/scale*scale rounded across a midpoint in fp32: never for these
    assert bool(same.all())
    exact = oracle.dequantize(q.cpu().numpy(), fmt, np.float32(scale.item()))
    assert np.array_equal(back.cpu().numpy(), exact.astype(np.float32))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_multi_tensor_amax_scale_and_cast_equal_the_oracle_and_the_single_tensor_calls(dtype):
    """fp8_amax_scale_multi / fp8_quantize_multi: up to four tensors of one element type per launch,
    each with its own format; amax, scale and bytes against the oracle (and thereby the single-tensor
    entry points), twice in a row on one workspace (the tickets must come back to zero), with sizes
    from one workgroup's share to many, ragged tails, specials; then the cases that are served
    tensor by tensor inside the call (an empty tensor, one that is not 16-byte aligned)."""
    rng = np.random.default_rng(23)
    fmts = [fp8.FP8_E4M3, fp8.FP8_E5M2, fp8.FP8_E5M2, fp8.FP8_E4M3]
    ws = torch.zeros(4 * fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
    for sizes in ([1 << 21, 300_007], [70_001, 1 << 22, 17, 1_000_000], [5, 9]):
        count = len(sizes)
        hs = []
        for k, n in enumerate(sizes):
            x = (rng.standard_normal(n) * np.float32(10.0 ** (k - 1))).astype(np.float32)
            if n > 1000:
                x[rng.integers(0, n, 4)] = [0.0, -0.0, 1e-30, -3e4 * 10.0 ** k]
            hs.append(x if dtype == "f32" else synth.to_bf16_bits(x))
        ds = [to_dev(h) for h in hs]
        amax = torch.full((count,), -1.0, device="cuda")
        scale = torch.full((count,), -1.0, device="cuda")
        qs = [torch.full((n,), 0xAA, dtype=torch.uint8, device="cuda") for n in sizes]
        for rep in range(2):
            fp8.fp8_amax_scale_multi(ds, fmts[:count], amax, scale, ws)
            fp8.fp8_quantize_multi(ds, fmts[:count], scale, qs)
            torch.cuda.synchronize()
            for k in range(count):
                a = oracle.amax(hs[k])
                sc = oracle.scale_from_amax(a, fmts[k])
                assert amax[k].item() == a and np.float32(scale[k].item()) == sc, (sizes, k, rep)
                want = oracle.quantize(hs[k], fmts[k], sc)
                got = qs[k].cpu().numpy()
                assert np.array_equal(got, want), (sizes, k, rep, int(np.count_nonzero(got != want)))
    # tensor-by-tensor service inside the call: an empty tensor and an unaligned one among aligned ones
    base = to_dev((rng.standard_normal(200_001)).astype(np.float32) if dtype == "f32" else synth.to_bf16_bits(rng.standard_normal(200_001).astype(np.float32)))
    odd = base[1:]                                                    # 4 or 2 bytes off a 16-byte boundary
    empty = torch.empty(0, dtype=base.dtype, device="cuda")
    big = to_dev(np.full(40_000, 3.0, dtype=np.float32) if dtype == "f32" else synth.to_bf16_bits(np.full(40_000, 3.0, dtype=np.float32)))
    xs = [big, empty, odd]
    amax = torch.full((3,), -1.0, device="cuda")
    scale = torch.full((3,), -1.0, device="cuda")
    qs = [torch.full((t.numel(),), 0xAA, dtype=torch.uint8, device="cuda") for t in xs]
    fp8.fp8_amax_scale_multi(xs, [fp8.FP8_E4M3] * 3, amax, scale, ws)
    fp8.fp8_quantize_multi(xs, [fp8.FP8_E4M3] * 3, scale, qs)
    torch.cuda.synchronize()
    assert amax[0].item() == 3.0 and amax[1].item() == 0.0 and scale[1].item() == 1.0
    ho = odd.cpu().view(torch.int16).numpy().view(np.uint16) if dtype == "bf16" else odd.cpu().numpy()
    a = oracle.amax(ho)
    assert amax[2].item() == a
    assert np.array_equal(qs[2].cpu().numpy(), oracle.quantize(ho, fp8.FP8_E4M3, oracle.scale_from_amax(a, fp8.FP8_E4M3)))
    assert np.array_equal(qs[0].cpu().numpy(), np.full(40_000, oracle.encode(fp8.FP8_E4M3, 448.0), dtype=np.uint8))
    for t in range(4):                                                # the counters' part of every tensor's workspace
        lo = t * fp8.FP8_AMAX_WORKSPACE_BYTES // 4
        assert int(ws[lo:lo + 32 * 33].abs().sum().item()) == 0, "a counter was left non-zero"
    rc = fp8.lib().fp8_amax_scale_multi(fp8.FP8_MULTI_MAX + 1, None, None, 0, None, amax.data_ptr(), None, ws.data_ptr(), None)
    assert rc == fp8.FP8_ERR_INVALID_ARG and "count" in fp8.binding.fp8_last_error()
