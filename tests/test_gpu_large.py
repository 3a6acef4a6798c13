"""GPU parity at sizes whose element counts and byte offsets do not fit 32 bits."""
import numpy as np
import pytest
import torch

import oracle
import paper_2209_05433_amd as fp8
from gpu_util import out_to_f64

pytestmark = pytest.mark.gpu

E4M3, E5M2 = fp8.FP8_E4M3, fp8.FP8_E5M2


def test_cast_and_amax_beyond_2_to_31_elements():
    """2^31 + 4101 bf16 elements (4.3 GB in, 2.1 GB out): windows at the start, around the 2^31 and
    2^32-byte marks and at the (ragged) end are compared with the oracle bit for bit; a planted
    maximum in the last element must be found."""
    n = (1 << 31) + 4101
    g = torch.Generator(device="cuda")
    g.manual_seed(31)
    x = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    step = 1 << 28
    for lo in range(0, n, step):                      # filled in pieces: no fp32 temporary of the full size
        hi = min(n, lo + step)
        x[lo:hi] = torch.randn(hi - lo, device="cuda", generator=g).to(torch.bfloat16)
    x[n - 1] = -768.0
    amax = torch.zeros(1, device="cuda")
    scale = torch.zeros(1, device="cuda")
    q = torch.empty(n, dtype=torch.uint8, device="cuda")
    fp8.fp8_amax(x, amax)
    fp8.fp8_scale_from_amax(amax, E4M3, scale)
    fp8.fp8_quantize_dscale(x, E4M3, scale, q)
    q2 = torch.empty(n, dtype=torch.uint8, device="cuda")
    amax2 = torch.zeros(1, device="cuda")
    fp8.fp8_quantize_amax(x, E4M3, scale, q2, amax2)
    torch.cuda.synchronize()
    assert amax.item() == 768.0 and amax2.item() == 768.0
    s = oracle.scale_from_amax(np.float32(768.0), oracle.E4M3)
    assert np.float32(scale.item()) == s
    w = 1 << 20
    for lo in (0, (1 << 30) - w // 2, (1 << 31) - w // 2, n - w):     # 2^30 elements = 2^31 bytes of input; 2^31 elements = 2^32 bytes
        hi = min(n, lo + w)
        xs = x[lo:hi].cpu().view(torch.int16).numpy().view(np.uint16)
        want = oracle.quantize(xs, oracle.E4M3, s)
        assert np.array_equal(q[lo:hi].cpu().numpy(), want), "cast differs in the window at %d" % lo
        assert np.array_equal(q2[lo:hi].cpu().numpy(), want), "single-pass cast differs in the window at %d" % lo
    assert torch.equal(q, q2)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_cast_of_an_output_beyond_the_memory_side_cache(dtype):
    """From 384 MiB of output on the casts store non-temporally and from many short runs: 384 Mi + 37
    elements (ragged end, both input types), E5M2, every byte against the oracle in windows, the
    single-pass cast against the plain one on everything."""
    n = (384 << 20) + 37
    g = torch.Generator(device="cuda")
    g.manual_seed(384)
    x = torch.empty(n, dtype=dtype, device="cuda")
    step = 1 << 27
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        x[lo:hi] = (torch.randn(hi - lo, device="cuda", generator=g) * 3.0).to(dtype)
    scale = torch.full((1,), 100.0, device="cuda")
    q = torch.empty(n, dtype=torch.uint8, device="cuda")
    q2 = torch.empty(n, dtype=torch.uint8, device="cuda")
    amax2 = torch.zeros(1, device="cuda")
    fp8.fp8_quantize_dscale(x, E5M2, scale, q)
    fp8.fp8_quantize_amax(x, E5M2, scale, q2, amax2)
    torch.cuda.synchronize()
    assert torch.equal(q, q2)
    assert amax2.item() == x.abs().max().item()
    w = 1 << 21
    for lo in (0, n // 3, n - w):
        xs = x[lo:lo + w].cpu()
        xs = xs.numpy() if dtype == torch.float32 else xs.view(torch.int16).numpy().view(np.uint16)
        want = oracle.quantize(xs, oracle.E5M2, np.float32(100.0))
        assert np.array_equal(q[lo:lo + w].cpu().numpy(), want), "cast differs in the window at %d" % lo


def test_gemm_with_operand_and_output_offsets_beyond_32_bits():
    """A of 65536 x 65536 bytes (4 GiB: row offsets pass 2^32) against a narrow B; and a product with
    2^31 outputs (65536 x 32768, 4 GiB of bf16: output offsets pass 2^32).  Sampled outputs, the last
    rows and columns included, against the oracle."""
    rng = np.random.default_rng(5)

    def codes(shape, seed):
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        mag = torch.randint(0, 0x60, shape, dtype=torch.uint8, device="cuda", generator=g)
        return mag | (torch.randint(0, 2, shape, dtype=torch.uint8, device="cuda", generator=g) << 7)

    # (1) long rows of A
    M, N, K = 65536, 256, 65536
    A, B = codes((M, K), 1), codes((K, N), 2)
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    pi = np.concatenate([[0, M - 1, M - 1, 40000], rng.integers(0, M, 60)]).astype(np.int64)
    pj = np.concatenate([[0, N - 1, 0, 17], rng.integers(0, N, 60)]).astype(np.int64)
    rows = torch.from_numpy(np.unique(pi)).cuda()
    A_rows = A[rows].cpu().numpy()                     # only the sampled rows travel to the host
    B_host = B.cpu().numpy()
    ridx = np.searchsorted(np.unique(pi), pi)
    S, T = oracle.gemm_points(A_rows, oracle.E4M3, B_host, oracle.E4M3, ridx, pj)
    for flags, rel in ((0, 2.0 ** -20), (fp8.FP8_GEMM_MFMA8, 2.0 ** -10)):
        fp8.fp8_gemm_ex(A, E4M3, 0, B, E4M3, 0, C, 2.0, 4.0, flags)
        torch.cuda.synchronize()
        got = C[torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda()].cpu().numpy().astype(np.float64)
        c_ref = S / 8.0
        assert np.all(np.abs(got - c_ref) <= rel * np.abs(T) / 8.0 + 0.5 * oracle.ulp(c_ref, oracle.F32)), flags
    del A, B, C

    # (2) 2^31 outputs
    M, N, K = 65536, 32768, 128
    A, B = codes((M, K), 3), codes((K, N), 4)
    C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    D = torch.empty((M, N), dtype=torch.uint8, device="cuda")
    one = torch.ones(1, device="cuda")
    pi = np.concatenate([[0, M - 1, M - 1, 0, 32768, 32767], rng.integers(0, M, 300)]).astype(np.int64)
    pj = np.concatenate([[0, N - 1, 0, N - 1, 0, N - 1], rng.integers(0, N, 300)]).astype(np.int64)
    S, T = oracle.gemm_points(A.cpu().numpy(), oracle.E4M3, B.cpu().numpy(), oracle.E4M3, pi, pj)
    ti, tj = torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda()
    fp8.fp8_gemm(A, E4M3, 1.0, B, E4M3, 1.0, C)
    fp8.fp8_gemm_fused(A, E4M3, 0, B, E4M3, 0, D, fp8.FP8_OUT_E5M2, one, one, None, None)
    torch.cuda.synchronize()
    assert np.all(np.abs(out_to_f64(C[ti, tj]) - S) <= 2.0 ** -20 * np.abs(T) + 0.5 * oracle.ulp(S, oracle.BF16))
    # K = 128 products of values with 4-bit significands: the sums are exact in fp32, the FP8 byte is the oracle's
    assert np.array_equal(D[ti, tj].cpu().numpy(), oracle.quantize(S.astype(np.float32), oracle.E5M2, 1.0))
