"""Seeded synthetic inputs shared by the oracle-side tests and the GPU-side tests/bench.

This module draws random tensors with the shapes and value distributions of the five
benchmark workloads (transformer-layer GEMMs and one large cast) and nothing else: it
contains no FP8 arithmetic, no scaling and no matrix multiply.  bfloat16 tensors are
returned as ``uint16`` arrays holding the bit patterns (numpy has no bfloat16); the
rounding from float32 is torch's CPU cast, a library routine.

Streams are reproducible and independent of the number of worker threads: a tensor is
cut into fixed chunks of ``CHUNK`` elements, chunk ``c`` of the tensor with seed ``s``
is drawn from ``numpy.random.Philox(key=s, counter=c << 64)``.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

BASE_SEED = 220905433
CHUNK = 1 << 22


def tensor_seed(config: int, which: int) -> int:
    """Seed of tensor ``which`` (0 = A or x, 1 = B) of benchmark config 1..5."""
    return BASE_SEED + 10 * config + which


def _workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _chunk_rng(seed: int, c: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=seed, counter=[0, 0, c, 0]))


def _fill(n: int, seed: int, draw) -> np.ndarray:
    """float32 vector of n elements; draw(rng, m) returns m float32 samples."""
    out = np.empty(n, dtype=np.float32)
    nchunks = (n + CHUNK - 1) // CHUNK

    def job(c):
        lo = c * CHUNK
        hi = min(n, lo + CHUNK)
        out[lo:hi] = draw(_chunk_rng(seed, c), hi - lo)

    if nchunks <= 1:
        for c in range(nchunks):
            job(c)
    else:
        with ThreadPoolExecutor(_workers()) as ex:
            list(ex.map(job, range(nchunks)))
    return out


def normal(n: int, seed: int, std: float = 1.0) -> np.ndarray:
    std32 = np.float32(std)
    return _fill(n, seed, lambda g, m: g.standard_normal(m, dtype=np.float32) * std32)


def normal_with_outliers(n: int, seed: int, p: float = 1e-3, factor: float = 1000.0) -> np.ndarray:
    """N(0,1) with a Bernoulli(p) subset multiplied by ``factor`` (in float32)."""
    def draw(g, m):
        x = g.standard_normal(m, dtype=np.float32)
        hit = g.random(m, dtype=np.float32) < np.float32(p)
        x[hit] *= np.float32(factor)
        return x
    return _fill(n, seed, draw)


def laplace(n: int, seed: int, b: float) -> np.ndarray:
    """Laplace(0, b) by the inverse CDF of a seeded uniform."""
    def draw(g, m):
        u = g.random(m, dtype=np.float64) - 0.5
        x = -b * np.sign(u) * np.log1p(-2.0 * np.abs(u))
        return x.astype(np.float32)
    return _fill(n, seed, draw)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 (torch CPU cast, round to nearest even) -> uint16 bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32 (for inspection only)."""
    return (h.astype(np.uint32) << 16).view(np.float32)


# ---------------------------------------------------------------------------------------
# The five workloads.  Sizes are parameters so that tests can take scaled-down versions
# with the same distributions and structure; defaults are the benchmark sizes.
# ---------------------------------------------------------------------------------------

def config1(M=256, N=256, K=256):
    """fp32 A (M x K) and B (K x N), i.i.d. N(0,1)."""
    A = normal(M * K, tensor_seed(1, 0)).reshape(M, K)
    B = normal(K * N, tensor_seed(1, 1)).reshape(K, N)
    return A, B


def config2(n=1 << 28):
    """bf16 vector, N(0,1) with 0.1 % of the entries multiplied by 1000."""
    return to_bf16_bits(normal_with_outliers(n, tensor_seed(2, 0)))


def config3(M=4096, N=6144, K=2048, n_outlier_channels=4):
    """bf16 activations N(0,1) with a few K-channels x100, bf16 weights N(0, 0.02)."""
    A = normal(M * K, tensor_seed(3, 0)).reshape(M, K)
    ch = np.random.Generator(np.random.Philox(key=tensor_seed(3, 0) + 5)).choice(
        K, size=min(n_outlier_channels, K), replace=False)
    A[:, ch] *= np.float32(100.0)
    B = normal(K * N, tensor_seed(3, 1), 0.02).reshape(K, N)
    return to_bf16_bits(A), to_bf16_bits(B)


def config4(M=8192, N=49152, K=12288):
    """bf16 activations N(0,1), bf16 weights N(0, 0.006)."""
    A = to_bf16_bits(normal(M * K, tensor_seed(4, 0))).reshape(M, K)
    B = to_bf16_bits(normal(K * N, tensor_seed(4, 1), 0.006)).reshape(K, N)
    return A, B


def config5(M=8192, N=12288, K=49152):
    """bf16 output gradients Laplace(0, 1e-5), bf16 weights N(0, 0.006)."""
    A = to_bf16_bits(laplace(M * K, tensor_seed(5, 0), 1e-5)).reshape(M, K)
    B = to_bf16_bits(normal(K * N, tensor_seed(5, 1), 0.006)).reshape(K, N)
    return A, B
