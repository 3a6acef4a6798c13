"""GPU parity of fp8_gemm_splitk_static, the entry point that allocates nothing (its slices' sums go
to a device array inside the library), against fp8_gemm_splitk with a caller-supplied workspace:
identical bits, on two calls in a row of which the second is smaller (what the first left in the
array must not enter the second), and a clear error beyond the array's size."""
import numpy as np
import pytest
import torch

import oracle
import paper_2209_05433_amd as fp8
from gpu_util import to_dev, out_to_f64

pytestmark = pytest.mark.gpu

E4M3, E5M2 = fp8.FP8_E4M3, fp8.FP8_E5M2


def codes(rng, shape, top):
    return rng.integers(0, top + 1, size=shape).astype(np.uint8) | (rng.integers(0, 2, size=shape).astype(np.uint8) << 7)


def both(dA, tA, dB, tB, M, N, K, dtype, sA, sB, flags, splits):
    need = fp8.fp8_gemm_splitk_workspace_size(M, N, K, tA, tB, splits)
    ws = torch.full((max(need, 16),), 0xFF, dtype=torch.uint8, device="cuda")
    C_ws = torch.full((M, N), 5.0, dtype=dtype, device="cuda")
    C_st = torch.full((M, N), 6.0, dtype=dtype, device="cuda")
    fp8.fp8_gemm_splitk(dA, E5M2, tA, dB, E4M3, tB, C_ws, sA, sB, ws, flags, splits)
    fp8.fp8_gemm_splitk_static(dA, E5M2, tA, dB, E4M3, tB, C_st, sA, sB, flags, splits)
    torch.cuda.synchronize()
    return C_ws, C_st, need


def test_static_scratch_gives_the_bits_of_the_workspace_form_on_two_calls_in_a_row():
    rng = np.random.default_rng(404)
    # first a large problem (16 slices of 1024 x 1024: the whole 64 MiB array), then a small ragged one
    cases = [(1024, 1024, 16384, 1, 0, torch.float32, 0), (300, 200, 64 * 37, 0, 1, torch.bfloat16, 5)]
    for flags in (0, fp8.FP8_GEMM_MFMA8):
        for (M, N, K, tA, tB, dtype, splits) in cases:
            A, B = codes(rng, (M, K), 0x4F), codes(rng, (K, N), 0x6F)
            dA = to_dev(np.ascontiguousarray(A.T) if tA else A)
            dB = to_dev(np.ascontiguousarray(B.T) if tB else B)
            C_ws, C_st, need = both(dA, tA, dB, tB, M, N, K, dtype, 3.0, 0.5, flags, splits)
            assert need > 0 and need <= fp8.FP8_SPLITK_STATIC_BYTES
            assert torch.equal(C_ws, C_st), "%d outputs differ" % int((C_ws != C_st).sum())
            # and both are the product, to the bound of the GEMM
            rows = np.array([0, M // 2, M - 1])
            S, T = oracle.gemm_rows(A, E5M2, B, E4M3, rows)
            c_ref, alpha = oracle.unscale(S, 3.0, 0.5)
            out = oracle.F32 if dtype == torch.float32 else oracle.BF16
            bound = (2.0 ** -10 if flags else 2.0 ** -20) * alpha * T + 0.5 * oracle.ulp(c_ref, out)
            assert np.all(np.abs(out_to_f64(C_st[torch.from_numpy(rows).cuda()]) - c_ref) <= bound)


def test_the_library_choice_is_cut_down_to_the_array_and_explicit_requests_beyond_it_are_refused():
    rng = np.random.default_rng(405)
    M, N, K = 2048, 1024, 8192                       # 32 tiles: the library's choice is 8 slices = 64 MiB, exactly the array
    A, B = codes(rng, (M, K), 0x4F), codes(rng, (K, N), 0x6F)
    dA, dB = to_dev(A), to_dev(B)
    C_ws, C_st, need = both(dA, 0, dB, 0, M, N, K, torch.float32, 1.0, 1.0, 0, 0)
    assert need == 8 * M * N * 4 == fp8.FP8_SPLITK_STATIC_BYTES and torch.equal(C_ws, C_st)
    M2 = 2304                                        # 36 tiles: 7 slices would need 66 MiB; the static form takes 7 -> what fits
    A2 = codes(rng, (M2, K), 0x4F)
    dA2 = to_dev(A2)
    C = torch.empty((M2, N), dtype=torch.float32, device="cuda")
    fp8.fp8_gemm_splitk_static(dA2, E5M2, 0, dB, E4M3, 0, C, 1.0, 1.0, 0, 0)
    torch.cuda.synchronize()
    rows = np.array([0, 1000, M2 - 1])
    S, T = oracle.gemm_rows(A2, E5M2, B, E4M3, rows)
    assert np.all(np.abs(out_to_f64(C[torch.from_numpy(rows).cuda()]) - S) <= 2.0 ** -20 * T + 0.5 * oracle.ulp(S, oracle.F32))
    C.fill_(7.0)
    with pytest.raises(fp8.Fp8Error) as e:
        fp8.fp8_gemm_splitk_static(dA2, E5M2, 0, dB, E4M3, 0, C, 1.0, 1.0, 0, 8)
    assert e.value.status == fp8.FP8_ERR_UNSUPPORTED and "static scratch array holds 67108864" in str(e.value)
    torch.cuda.synchronize()
    assert bool((C == 7.0).all()), "a refused call must not launch anything"
