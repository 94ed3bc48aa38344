"""CPU-side seeded inputs (numpy, PCG64) for the workloads whose expected values are stored as
fixtures: the generator has to give the same arrays on every machine, which a device generator
does not promise.  Like ``workloads.py`` this module only draws random matrices and rounds them
to the storage format: none of the method's arithmetic (statistics, roots, products, rotations)
lives here.  It imports nothing from the package, so a script that must not load the HIP library
can load this file by path.

Every stream is ``numpy.random.Generator(PCG64(SeedSequence([20260516, cfg, block, step])))``.
"""
from __future__ import annotations

import numpy as np

SEED0 = 20260516


def rng(cfg: int, block: int, step: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([SEED0, cfg, block, step])))


def haar(g: np.random.Generator, n: int) -> np.ndarray:
    """Orthogonal matrix from the QR of a Gaussian, column signs fixed by diag(R) > 0."""
    a = g.standard_normal((n, n))
    q, r = np.linalg.qr(a)
    return q * np.sign(np.diag(r))


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (ties to even), returned as float64.
    One rounding, straight from float64: 8 significant bits.  Normal range only."""
    m, e = np.frexp(np.asarray(x, dtype=np.float64))
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are exactly representable in bfloat16."""
    b = np.asarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(b & np.uint32(0xFFFF)), "value is not a bfloat16"
    return (b >> np.uint32(16)).astype(np.uint16)


def logspaced_sigma(r: int, decades: float) -> np.ndarray:
    """sigma_i log-spaced from 1 down to 10^-decades."""
    return 10.0 ** (-decades * np.arange(r, dtype=np.float64) / max(r - 1, 1))


def logspaced_block(cfg: int, block: int, n: int = 4096, decades: float = 8.0) -> np.ndarray:
    """G = bf16(U diag(sigma) V^T), U and V Haar, sigma log-spaced over `decades` decades
    (the ill-conditioned stress workload: 4096 x 4096, 8 decades).  float64 array of bf16 values."""
    g = rng(cfg, block)
    U = haar(g, n)
    V = haar(g, n)
    return round_bf16((U * logspaced_sigma(n, decades)) @ V.T)


def sample_rows(cfg: int, block: int, side: int, n: int, count: int) -> np.ndarray:
    """Sorted seeded choice of `count` distinct row indices below n (side 0 = L, 1 = R)."""
    g = rng(cfg, block, 1000 + side)
    return np.sort(g.choice(n, size=count, replace=False))
