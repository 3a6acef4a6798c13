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


class cast_path:
    """Context manager selecting the cast implementation of the library (bits | cvt)."""
    def __init__(self, name):
        self.name = name

    def __enter__(self):
        self.old = os.environ.get("FP8MM_CAST_PATH")
        os.environ["FP8MM_CAST_PATH"] = self.name

    def __exit__(self, *exc):
        if self.old is None:
            os.environ.pop("FP8MM_CAST_PATH", None)
        else:
            os.environ["FP8MM_CAST_PATH"] = self.old


def report_byte_mismatch(x_bits, got, want, limit=8):
    bad = np.flatnonzero(got != want)
    lines = ["%d of %d bytes differ" % (bad.size, got.size)]
    for i in bad[:limit]:
        lines.append("  elem %d input bits 0x%x got 0x%02x want 0x%02x" % (i, int(x_bits[i]), got[i], want[i]))
    return "\n".join(lines)
