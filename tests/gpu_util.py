"""Helpers shared by the GPU parity tests: host arrays <-> device buffers, mismatch reports."""
import os

import numpy as np
import torch


def to_dev(a: np.ndarray) -> torch.Tensor:
    """float32 stays float32, uint16 is taken as bfloat16 bit patterns, uint8 stays bytes."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def bf16_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.cpu().view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f64(h: np.ndarray) -> np.ndarray:
    return (h.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def out_to_f64(C: torch.Tensor) -> np.ndarray:
    if C.dtype == torch.bfloat16:
        return bf16_bits_to_f64(bf16_to_bits(C))
    return C.cpu().numpy().astype(np.float64)


class knob:
    """Context manager: one tuning knob of the library set to a value, restored on exit."""
    def __init__(self, which, value):
        self.which, self.value = which, value

    def __enter__(self):
        import paper_2209_05433_amd as fp8
        self.old = fp8.fp8_set_knob(self.which, self.value)

    def __exit__(self, *exc):
        import paper_2209_05433_amd as fp8
        fp8.fp8_set_knob(self.which, self.old)


def cast_path(name):
    """Selects the cast implementation of the library (bits | cvt)."""
    import paper_2209_05433_amd as fp8
    return knob(fp8.FP8_KNOB_CAST_PATH, {"cvt": 0, "bits": 1}[name])


def report_byte_mismatch(x_bits, got, want, limit=8):
    bad = np.flatnonzero(got != want)
    lines = ["%d of %d bytes differ" % (bad.size, got.size)]
    for i in bad[:limit]:
        lines.append("  elem %d input bits 0x%x got 0x%02x want 0x%02x" % (i, int(x_bits[i]), got[i], want[i]))
    return "\n".join(lines)


def freivalds_blocks(C, Aq, fmtA, Bq, fmtB, sA, sB, out_dtype, rel=2.0 ** -20, seeds=(1, 2), block=256, label=""):
    """Whole-matrix acceptance of a GEMM result too large for the element-by-element reference:
    for seeded +-1 vectors r and every block of `block` consecutive columns,
        | sum_{j in block} r_j C[i, j]  -  alpha * sum_{j in block} r_j S[i, j] |
            <=  sum_{j in block} ( rel * alpha * T[i, j] + ulp_out(C[i, j]) / 2 )
    which every C that meets the element bound meets (the half-ulps are taken at |C| (1 + 2^-6), so
    that an output that was rounded across a power of two is still covered).  Every output enters
    one such sum per vector; a sum covers few enough outputs for a single wrong one to stand out.
    The left sums of the device result are formed here in double precision; the reference sums
    come from oracle.gemm_block_sums.  sA / sB: per-tensor factors (alpha = 1 / (sA sB)).  Returns
    the worst error / bound."""
    import oracle
    M, N = C.shape
    alpha = 1.0 / (float(np.float32(sA)) * float(np.float32(sB)))
    starts = np.arange(0, N, block)
    rs, refs = [], []
    for seed in seeds:
        r = np.random.default_rng(seed).choice([-1.0, 1.0], N)
        rs.append(r)
        refs.append(oracle.gemm_block_sums(Aq, fmtA, Bq, fmtB, r, block))
    worst = 0.0
    step = max(1, (1 << 25) // N)
    for i0 in range(0, M, step):
        c = out_to_f64(C[i0:i0 + step])
        assert np.all(np.isfinite(c)), label + ": non-finite outputs in rows %d.." % i0
        half_ulps = np.add.reduceat(0.5 * oracle.ulp(c * (1.0 + 2.0 ** -6), out_dtype), starts, axis=1)
        for r, (SR, TR) in zip(rs, refs):
            got = np.add.reduceat(c * r, starts, axis=1)
            bound = (rel + 1e-13) * alpha * TR[i0:i0 + step] + half_ulps
            err = np.abs(got - alpha * SR[i0:i0 + step])
            ratio = err / bound
            w = np.unravel_index(np.argmax(ratio), ratio.shape)
            assert np.all(err <= bound), "%s: block sums of row %d, columns %d..: err/bound %.3g" % (
                label, i0 + w[0], w[1] * block, ratio[w])
            worst = max(worst, float(ratio.max()))
    return worst
