"""Seeded synthetic inputs for the u8 x s8 -> s32 GEMM workloads.

This module only draws random bytes and shapes.  It holds none of the method's
arithmetic and is the one module both the CPU oracle's tests and the HIP path's
tests/benchmark use, so that both sides see the same bytes.

Conventions: A is uint8 (M, K) row-major; B is int8 of shape (N, K), i.e. the
column-major K x N operand (the paper's [N x K] storage, Sec. 2.1).
The shapes stand in for "DNN-shaped matrices": the paper's own problem-size
list is only in a figure that did not survive, and its models are private.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 191000178


def rng_for(config: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config + sub))


@dataclass
class Problem:
    name: str
    A: np.ndarray            # (M, K) uint8
    B: np.ndarray            # (N, K) int8  (column-major K x N)
    za: int = 0
    zb: int = 0
    scale: Optional[float] = None   # requantise-to-u8 variant when not None
    zc: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def M(self): return self.A.shape[0]
    @property
    def N(self): return self.B.shape[0]
    @property
    def K(self): return self.A.shape[1]


def uniform_u8(rng, M, K):
    return rng.integers(0, 256, size=(M, K), dtype=np.uint8)


def uniform_s8(rng, N, K):
    return rng.integers(-128, 128, size=(N, K), dtype=np.int8)


def gaussian_u8(rng, M, K, mean=128.0, sd=40.0):
    return np.clip(np.rint(rng.normal(mean, sd, size=(M, K))), 0, 255).astype(np.uint8)


def gaussian_s8(rng, N, K, sd=30.0):
    return np.clip(np.rint(rng.normal(0.0, sd, size=(N, K))), -127, 127).astype(np.int8)


def tiny():
    """Config 1: M=64, N=64, K=256, uniform operands, zero-points 0."""
    rng = rng_for(1)
    return Problem("tiny_64x64x256", uniform_u8(rng, 64, 256), uniform_s8(rng, 64, 256))


BERT_FC_SHAPES = ((768, 768), (3072, 768), (768, 3072))   # (N, K)


def bert_fc(index: int, M: int = 1024):
    """Config 2: 1024 tokens; clipped-Gaussian activations with zero-point 128,
    Gaussian weights; also run with the requantise-to-u8 epilogue."""
    N, K = BERT_FC_SHAPES[index]
    rng = rng_for(2, index)
    scale = 0.00096 if K == 768 else 0.00048
    return Problem(f"bert_fc_{M}x{N}x{K}", gaussian_u8(rng, M, K), gaussian_s8(rng, N, K),
                   za=128, zb=0, scale=float(np.float32(scale)), zc=128)


def skinny(M: int, N: int = 4096, K: int = 1024, n_a: int = 16):
    """Config 3: LSTM-gate-like skinny GEMM; one B reused, a pool of n_a inputs A."""
    rng = rng_for(3, M)
    B = uniform_s8(rng, N, K)
    As = [uniform_u8(rng, M, K) for _ in range(n_a)]
    return [Problem(f"skinny_{M}x{N}x{K}_a{t}", As[t], B) for t in range(n_a)]


def large_square(n: int = 8192):
    """Config 4: M=N=K=8192 uniform operands, zero-points 0."""
    rng = rng_for(4)
    return Problem(f"square_{n}", uniform_u8(rng, n, n), uniform_s8(rng, n, n))


def _log_uniform_dim(rng, dmax):
    u = rng.random()
    return int(min(dmax, max(1, int(np.floor(2.0 ** (u * np.log2(dmax + 1)))))))


def batched_shapes(count: int = 64, mmax: int = 2048, nmax: int = 4096, kmax: int = 4096, sub: int = 0):
    """Config 5 shapes and zero-points only (no matrices)."""
    rng = rng_for(5, sub)
    out = []
    for _ in range(count):
        M = _log_uniform_dim(rng, mmax)
        N = _log_uniform_dim(rng, nmax)
        K = _log_uniform_dim(rng, kmax)
        za = int(rng.integers(0, 256))
        zb = int(rng.integers(-8, 9))
        out.append((M, N, K, za, zb))
    return out


def batched(count: int = 64, mmax: int = 2048, nmax: int = 4096, kmax: int = 4096, sub: int = 0):
    """Config 5: independent GEMMs with log-uniform odd shapes and per-GEMM zero-points."""
    shapes = batched_shapes(count, mmax, nmax, kmax, sub)
    rng = rng_for(5, 500 + sub)
    probs = []
    for t, (M, N, K, za, zb) in enumerate(shapes):
        probs.append(Problem(f"batched{t}_{M}x{N}x{K}", uniform_u8(rng, M, K), uniform_s8(rng, N, K),
                             za=za, zb=zb))
    return probs
