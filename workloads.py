"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves BOTH the oracle-side and the GPU-side of every test and of
the benchmark, and therefore holds none of the method's arithmetic: only shapes,
seeds, random draws and the (exact) bf16 rounding of inputs.  It imports neither
the oracle nor the product package.

Recipe: numpy.random.default_rng(seed).standard_normal(shape, dtype=float32),
tensors drawn in the order Q, K, V, dO (decode: q, k, v streams shaped
[T, B, H, feature]).  The paper's sequence shapes are kept (784 = 28x28 pixel
images and 32 dims per head, section 4.2.1; 3072 = 32x32x3 images, section
4.2.2; the N = 2^9..2^16 sweep on synthetic input with the batch scaled
inversely to N, section 4.1.2); the pixel / audio data themselves are replaced
by i.i.d. Gaussian values, because the cost of the path depends on shapes only.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    D: int
    M: int
    seed: int
    scale: float = 1.0      # multiplies Q, K and V (not dO)
    eps: float = 1e-6


CFG1 = Workload("cfg1_fwd_N256_D32", 1, 1, 256, 32, 32, 1001)
CFG2 = Workload("cfg2_mnist_B8_H8_N784_D32", 8, 8, 784, 32, 32, 1002)
CFG3 = Workload("cfg3_cifar_B4_H8_N3072_D64", 4, 8, 3072, 64, 64, 1003, scale=1.0 / 8.0)


def sweep_point(log2n: int) -> Workload:
    """Sequence-length sweep: B*N = 2^17 tokens, H = 8, D = M = 64."""
    assert 9 <= log2n <= 16
    n = 1 << log2n
    return Workload(f"sweep_N2^{log2n}_B{(1 << 17) // n}_H8_D64", (1 << 17) // n, 8, n, 64, 64,
                    1400 + log2n)


HEADLINE = sweep_point(16)          # B=2, H=8, N=65536, D=M=64: the metric's workload


@dataclass(frozen=True)
class DecodeWorkload:
    name: str
    B: int
    H: int
    D: int
    M: int
    T: int
    seed: int
    eps: float = 1e-6


CFG5 = DecodeWorkload("cfg5_decode_B64_H8_D64_T3072", 64, 8, 64, 64, 3072, 1005)


def qkvg(w: Workload, with_grad: bool = True):
    """float32 Q, K [B,H,N,D], V [B,H,N,M] and (optionally) dO [B,H,N,M]."""
    rng = np.random.default_rng(w.seed)
    Q = rng.standard_normal((w.B, w.H, w.N, w.D), dtype=np.float32)
    K = rng.standard_normal((w.B, w.H, w.N, w.D), dtype=np.float32)
    V = rng.standard_normal((w.B, w.H, w.N, w.M), dtype=np.float32)
    if w.scale != 1.0:
        s = np.float32(w.scale)
        Q *= s
        K *= s
        V *= s
    if not with_grad:
        return Q, K, V
    G = rng.standard_normal((w.B, w.H, w.N, w.M), dtype=np.float32)
    return Q, K, V, G


def decode_streams(w: DecodeWorkload, T: int | None = None):
    """float32 q, k [T,B,H,D] and v [T,B,H,M]: one token per head per step."""
    T = w.T if T is None else T
    rng = np.random.default_rng(w.seed)
    q = rng.standard_normal((T, w.B, w.H, w.D), dtype=np.float32)
    k = rng.standard_normal((T, w.B, w.H, w.D), dtype=np.float32)
    v = rng.standard_normal((T, w.B, w.H, w.M), dtype=np.float32)
    return q, k, v


def random_case(seed: int, B: int, H: int, N: int, D: int, M: int, scale: float = 1.0):
    """Free-form seeded case for edge-size tests."""
    return qkvg(Workload(f"case{seed}", B, H, N, D, M, seed, scale=scale))


def wide_range_case(seed: int, B: int, H: int, N: int, D: int, M: int, log2_spread: int = 10):
    """Seeded case whose elements differ widely in magnitude inside every tile: each element of
    the Gaussian Q, K, V, dO is multiplied by its own power of two, 2^k with k uniform in
    [-log2_spread, 0] for Q and K (the feature map saturates large inputs anyway) and in
    [-log2_spread, log2_spread] for V and dO."""
    q, k, v, g = random_case(seed, B, H, N, D, M)
    rng = np.random.default_rng(seed + 7919)
    out = []
    for x, lo, hi in ((q, -log2_spread, 0), (k, -log2_spread, 0), (v, -log2_spread, log2_spread),
                      (g, -log2_spread, log2_spread)):
        e = rng.integers(lo, hi + 1, size=x.shape)
        out.append(np.ldexp(x, e).astype(np.float32))
    return tuple(out)


# ---- exact bf16 rounding of inputs (round to nearest, ties to even) -----------------------

def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array with every value rounded to the nearest bfloat16 (ties to
    even); the result is still float32 and exactly representable in bf16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    out = (r & 0xFFFFFFFF).astype(np.uint32).view(np.float32)
    nan = np.isnan(x)
    if nan.any():
        out = out.copy()
        out[nan] = np.float32(np.nan)
    return out.reshape(x.shape)


def bf16_bits(x_rounded: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an array already rounded by round_to_bf16."""
    x = np.ascontiguousarray(x_rounded, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return b.view(np.float32).reshape(bits.shape)
