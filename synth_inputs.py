"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module only draws random arrays and converts number formats.  It contains none of the
method's arithmetic (no factorization, no layer evaluation) and imports neither the GPU library
nor the CPU oracle, so both can be fed the very same arrays.

The paper trains ImageNet/CIFAR-10 models (ResNet-50/101/152, ViT); those datasets and weights
are not used here.  Throughput and correctness of a decomposed layer depend only on shapes,
dtypes and alignment, so arrays with the layer shapes of those networks and simple stated
distributions stand in for them.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 230903824


def rng_for(config: int, stream: int = 0) -> np.random.Generator:
    """One PCG64 stream per (config, stream) pair."""
    return np.random.Generator(np.random.PCG64([BASE_SEED + int(config), int(stream)]))


# ----------------------------------------------------------------------------- number formats
def bf16_bits(a) -> np.ndarray:
    """float -> bfloat16 bit patterns (uint16), round to nearest even."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f64(bits) -> np.ndarray:
    """bfloat16 bit patterns -> float64 (exact)."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_bf16(a) -> np.ndarray:
    """Values rounded to bfloat16 and widened back to float64."""
    return bf16_to_f64(bf16_bits(a))


def round_f32(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float32).astype(np.float64)


# ----------------------------------------------------------------------------- building blocks
def haar_orthogonal(n: int, rng: np.random.Generator) -> np.ndarray:
    """Random orthogonal matrix (Haar): Q of a Gaussian matrix, column signs fixed by diag(R)."""
    q, r = np.linalg.qr(rng.standard_normal((n, n)))
    return q * np.sign(np.diag(r))[None, :]


def gaussian(shape, rng: np.random.Generator, std: float = 1.0) -> np.ndarray:
    return rng.standard_normal(shape) * std


# ----------------------------------------------------------------------------- workloads
def config1_weight(n: int = 768, decay: float = 100.0, rng: np.random.Generator | None = None):
    """W = Q1 diag(sigma) Q2^T with sigma_i = exp(-i/decay), i = 0..n-1.  Returns (W, sigma)."""
    rng = rng or rng_for(1, 0)
    q1 = haar_orthogonal(n, rng)
    q2 = haar_orthogonal(n, rng)
    sigma = np.exp(-np.arange(n) / decay)
    return (q1 * sigma[None, :]) @ q2.T, sigma


def linear_weight(n_out: int, n_in: int, rng: np.random.Generator) -> np.ndarray:
    """W [out,in] ~ N(0, 1/fan_in)."""
    return gaussian((n_out, n_in), rng, std=1.0 / np.sqrt(n_in))


def direct_factors(n_out: int, n_in: int, r: int, rng: np.random.Generator):
    """Factor arrays drawn directly (U ~ N(0,1/r), V ~ N(0,1/in)) where a true SVD of a large
    weight would only cost time: the speed and the arithmetic of the layer do not depend on how
    the factors were obtained."""
    U = gaussian((n_out, r), rng, std=1.0 / np.sqrt(r))
    V = gaussian((r, n_in), rng, std=1.0 / np.sqrt(n_in))
    return U, V


def conv_weight(S: int, C: int, k: int, rng: np.random.Generator) -> np.ndarray:
    """W [S,k,k,C] ~ N(0, 1/(k*k*C))."""
    return gaussian((S, k, k, C), rng, std=1.0 / np.sqrt(k * k * C))


def direct_tucker_factors(S: int, C: int, k: int, r1: int, r2: int, rng: np.random.Generator):
    P1 = gaussian((r1, C), rng, std=1.0 / np.sqrt(C))
    G = gaussian((r2, k, k, r1), rng, std=1.0 / np.sqrt(k * k * r1))
    P2 = gaussian((S, r2), rng, std=1.0 / np.sqrt(r2))
    return P1, G, P2
