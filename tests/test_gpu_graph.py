"""The whole path (amax -> scale -> cast -> GEMM -> unscale, plus the fused variants) recorded once
into a HIP graph and replayed: no entry point allocates, synchronises or uses a memset node, so the
recorded launches must reproduce the eager results bit for bit on every replay, also after the
inputs have changed and with eager work in between."""
import numpy as np
import pytest
import torch

import oracle
import paper_2209_05433_amd as fp8
from workloads import synth
from gpu_util import to_dev, out_to_f64

pytestmark = pytest.mark.gpu

E4M3, E5M2 = fp8.FP8_E4M3, fp8.FP8_E5M2


def test_path_replayed_from_a_graph_matches_eager_and_oracle():
    M, N, K = 512, 768, 256
    dA = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    dB = torch.empty((K, N), dtype=torch.bfloat16, device="cuda")
    amax = torch.zeros(3, device="cuda")
    scale = torch.zeros(3, device="cuda")
    hist = torch.zeros(4, device="cuda")
    qA = torch.empty((M, K), dtype=torch.uint8, device="cuda")
    qAt = torch.empty((K, M), dtype=torch.uint8, device="cuda")
    qB = torch.empty((K, N), dtype=torch.uint8, device="cuda")
    C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    D = torch.empty((M, N), dtype=torch.uint8, device="cuda")
    W = torch.empty((K, N), dtype=torch.float32, device="cuda")       # A^T-shaped product: (K x M) x (M x N)
    W2, W3 = torch.empty_like(W), torch.empty_like(W)
    ws_amax = torch.zeros(fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
    ws_k = torch.empty(fp8.fp8_gemm_splitk_workspace_size(K, N, M, 0, 0, 2), dtype=torch.uint8, device="cuda")
    ws_multi = torch.zeros(2 * fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
    amax2, scale2 = torch.zeros(2, device="cuda"), torch.zeros(2, device="cuda")
    q2A, q2B = torch.empty_like(qA), torch.empty_like(qB)
    ws_one = torch.zeros(2 * fp8.FP8_AMAX_WORKSPACE_BYTES // 4, dtype=torch.int32, device="cuda")
    amax3, scale3 = torch.zeros(2, device="cuda"), torch.zeros(2, device="cuda")
    q3A, q3B, C3 = torch.empty_like(qA), torch.empty_like(qB), torch.empty_like(C)

    def step():
        fp8.fp8_amax(dA, amax[0:1])
        fp8.fp8_scale_from_amax(amax[0:1], E4M3, scale[0:1])
        fp8.fp8_quantize_transpose(dA, E4M3, scale[0:1], qA, qAt)
        fp8.fp8_scale_from_amax_history(hist, E4M3, scale[1:2])
        fp8.fp8_quantize_amax(dB, E4M3, scale[1:2], qB, hist[0:1])
        fp8.fp8_gemm_dscale(qA, E4M3, scale[0:1], qB, E4M3, scale[1:2], C)
        fp8.fp8_gemm_fused(qA, E4M3, 0, qB, E4M3, 0, D, fp8.FP8_OUT_E5M2, scale[0:1], scale[1:2], None, amax[2:3],
                           fp8.FP8_GEMM_MFMA8)
        fp8.fp8_gemm_ex(qAt, E4M3, 0, D, E5M2, 0, W, 1.0, 1.0)          # a second GEMM fed by the first one's FP8 output
        fp8.fp8_amax_scale(dB, E5M2, amax[1:2], scale[2:3], ws_amax)     # one-launch amax + scale (tickets in a workspace)
        fp8.fp8_gemm_splitk(qAt, E4M3, 0, D, E5M2, 0, W2, 1.0, 1.0, ws_k, 0, 2)     # the same product in two K slices
        fp8.fp8_gemm_splitk_static(qAt, E4M3, 0, D, E5M2, 0, W3, 1.0, 1.0, 0, 2)     # ... with the library's own scratch array
        fp8.fp8_amax_scale_multi((dA, dB), (E4M3, E5M2), amax2, scale2, ws_multi)     # both operands per launch
        fp8.fp8_quantize_multi((dA, dB), (E4M3, E5M2), scale2, (q2A, q2B))
        fp8.fp8_scaled_gemm(dA, E4M3, False, dB, E5M2, False, q3A, q3B, amax3, scale3, ws_one, C3)     # the whole path in one call

    def load(seed):
        a, b = synth.config3(M, N, K)
        rng = np.random.default_rng(seed)
        a = synth.to_bf16_bits(synth.bf16_bits_to_f32(a) * np.float32(rng.uniform(0.5, 2.0)))
        b = synth.to_bf16_bits(synth.bf16_bits_to_f32(b) * np.float32(rng.uniform(0.5, 2.0)) + np.float32(seed * 1e-3))
        dA.copy_(to_dev(a))
        dB.copy_(to_dev(b))
        return a, b

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (amax, scale, hist, qA, qAt, qB, C, D, W, W2, W3, amax2, scale2, q2A, q2B, amax3, scale3, q3A, q3B, C3)]

    load(0)
    hist.zero_()
    step()                                   # warm-up outside the capture (first launches set kernel attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for trial in range(4):
        a_bits, b_bits = load(trial + 1)
        hist.fill_(0.25 * (trial + 1))       # the history cell is overwritten by the step: reset it for both runs
        amax.fill_(-1.0)
        step()
        eager = snapshot()
        # unrelated eager work and a synchronisation between the replays
        junk = torch.randn(1 << 20, device="cuda").sum().item()
        hist.fill_(0.25 * (trial + 1))
        for t in (qA, qAt, qB, C, D):
            t.zero_()
        for t in (W, W2, W3, q2A, q2B, scale2, q3A, q3B, C3, scale3):
            t.zero_()
        amax3.fill_(-1.0)
        amax.fill_(-1.0)
        amax2.fill_(-1.0)
        graph.replay()
        replayed = snapshot()
        for e, r, name in zip(eager, replayed, "amax scale hist qA qAt qB C D W W2 W3 amax2 scale2 q2A q2B amax3 scale3 q3A q3B C3".split()):
            assert torch.equal(e.view(torch.uint8), r.view(torch.uint8)), "replay %d differs from eager in %s" % (trial, name)
        if trial == 0:                       # and eager is what the oracle says
            sA = oracle.scale_from_amax(oracle.amax(a_bits), oracle.E4M3)
            sB = oracle.scale_from_amax_history(np.full(4, 0.25, np.float32), oracle.E4M3)
            Aq, Bq = oracle.quantize(a_bits, oracle.E4M3, sA), oracle.quantize(b_bits, oracle.E4M3, sB)
            assert np.array_equal(eager[3].cpu().numpy(), Aq) and np.array_equal(eager[4].cpu().numpy(), Aq.T)
            assert np.array_equal(eager[5].cpu().numpy(), Bq)
            assert np.float32(eager[2][0].item()) == oracle.amax(b_bits)
            S, T = oracle.gemm_rows(Aq, oracle.E4M3, Bq, oracle.E4M3)
            c_ref, bound = oracle.gemm_bound(S, T, sA, sB, oracle.BF16)
            assert np.all(np.abs(out_to_f64(eager[6]) - c_ref) <= bound)
            assert torch.equal(eager[9], eager[10]) and np.float32(eager[0][1].item()) == oracle.amax(b_bits)
            assert np.float32(eager[1][2].item()) == oracle.scale_from_amax(oracle.amax(b_bits), oracle.E5M2)
            assert np.array_equal(eager[13].cpu().numpy(), Aq)              # the multi-tensor calls: A as above, B to E5M2
            assert np.array_equal(eager[14].cpu().numpy(), oracle.quantize(b_bits, oracle.E5M2, np.float32(eager[1][2].item())))
            assert torch.equal(eager[15], eager[11]) and torch.equal(eager[16], eager[12])      # one call = the multi calls
            assert torch.equal(eager[17], eager[13]) and torch.equal(eager[18], eager[14])
            S3, T3 = oracle.gemm_rows(Aq, oracle.E4M3, eager[14].cpu().numpy(), oracle.E5M2)
            c3_ref, bound3 = oracle.gemm_bound(S3, T3, np.float32(eager[12][0].item()), np.float32(eager[12][1].item()), oracle.BF16)
            assert np.all(np.abs(out_to_f64(eager[19]) - c3_ref) <= bound3)
