"""Seeded synthetic inputs shaped like the paper's workloads (OLMo / LLaMA-style 2-D weight
gradients, blocked at a maximum preconditioner dimension).  This module only draws random
matrices and lists shapes: none of the method's arithmetic (statistics, roots, products,
rotations) lives here, so the HIP path and the CPU oracle can both be fed from it.

All generators take a ``torch.Generator``-free integer seed and a device; the same seed on the
same device reproduces the same tensors.  Tests always hand both sides the very tensors that
were generated (downloaded once), so CPU/GPU generator differences never matter.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import torch

SEED0 = 20260516


def _gen(device, *key: int) -> torch.Generator:
    g = torch.Generator(device=device)
    s = SEED0
    for k in key:
        s = (s * 1000003 + int(k) + 12345) % (2 ** 62)
    g.manual_seed(s)
    return g


# --------------------------------------------------------------------------------- shapes

def llama_1b_matrices(d: int = 2048, layers: int = 22, ffn: int = 5632, vocab: int = 32000,
                      kv_dim: int = 256) -> List[Tuple[str, int, int]]:
    """2-D parameters of a 1.1B LLaMA-style model (rows x cols as stored: out x in)."""
    mats = []
    for l in range(layers):
        mats += [(f"l{l}.q", d, d), (f"l{l}.k", kv_dim, d), (f"l{l}.v", kv_dim, d), (f"l{l}.o", d, d),
                 (f"l{l}.gate", ffn, d), (f"l{l}.up", ffn, d), (f"l{l}.down", d, ffn)]
    mats += [("embed", vocab, d), ("lm_head", vocab, d)]
    return mats


def split_dim(d: int, B: int) -> List[int]:
    """Greedy split of one dimension into chunks of B with one remainder chunk last."""
    out = [B] * (d // B)
    if d % B:
        out.append(d % B)
    return out


def block_shapes(mats: Sequence[Tuple[str, int, int]], B: int) -> List[Tuple[int, int]]:
    """Every (row-chunk, col-chunk) pair of every matrix is an independent block."""
    blocks = []
    for _, r, c in mats:
        for m in split_dim(r, B):
            for n in split_dim(c, B):
                blocks.append((m, n))
    return blocks


def census(blocks: Sequence[Tuple[int, int]]):
    """(number of blocks by shape, number of factors by size, parameter count)."""
    by_shape, by_factor, params = {}, {}, 0
    for m, n in blocks:
        by_shape[(m, n)] = by_shape.get((m, n), 0) + 1
        by_factor[m] = by_factor.get(m, 0) + 1
        by_factor[n] = by_factor.get(n, 0) + 1
        params += m * n
    return by_shape, by_factor, params


# --------------------------------------------------------------------------------- matrices

def haar(n: int, device, *key: int, dtype=torch.float32, qr_on_host: bool = False) -> torch.Tensor:
    """Orthogonal matrix from the QR of a Gaussian, column signs fixed by diag(R) > 0.  With
    ``qr_on_host`` the Gaussian is drawn on the device as usual but factorised by the host's LAPACK
    (runs under hardware counters keep the device's solver library out of the process)."""
    g = _gen(device, 7, n, *key)
    a = torch.randn(n, n, generator=g, device=device, dtype=dtype)
    if qr_on_host:
        q, r = torch.linalg.qr(a.cpu())
        return (q * torch.sign(torch.diagonal(r))).contiguous().to(device)
    q, r = torch.linalg.qr(a)
    return (q * torch.sign(torch.diagonal(r))).contiguous()


def gaussian_block(m: int, n: int, std: float, device, *key: int, dtype=torch.float32) -> torch.Tensor:
    """G ~ N(0, std^2), e.g. the 128 x 128 fp32 single-block workload."""
    g = _gen(device, 1, m, n, *key)
    return (std * torch.randn(m, n, generator=g, device=device, dtype=torch.float32)).to(dtype)


def lowrank_block(m: int, n: int, device, *key: int, rank: int = 32, scale: float = 0.01,
                  noise: float = 1e-4, dtype=torch.bfloat16) -> torch.Tensor:
    """G = scale * Ua Ub^T + E with Gaussian rank-`rank` factors and N(0, noise^2) noise."""
    g = _gen(device, 2, m, n, *key)
    ua = torch.randn(m, rank, generator=g, device=device)
    ub = torch.randn(n, rank, generator=g, device=device)
    e = noise * torch.randn(m, n, generator=g, device=device)
    return (scale * (ua @ ub.T) + e).to(dtype)


def spectrum_block(U: torch.Tensor, V: torch.Tensor, sigma: torch.Tensor, device, *key: int,
                   rms: float | None = 0.01, dtype=torch.bfloat16) -> torch.Tensor:
    """G = U[:, p] diag(sigma) (V[:, q] * s)^T with a seeded column permutation / sign flips of the
    template bases, optionally rescaled to a target RMS entry."""
    m, n = U.shape[0], V.shape[0]
    r = min(m, n)
    g = _gen(device, 3, m, n, *key)
    pu = torch.randperm(m, generator=g, device=device)[:r]
    pv = torch.randperm(n, generator=g, device=device)[:r]
    sg = torch.randint(0, 2, (r,), generator=g, device=device).to(U.dtype) * 2 - 1
    G = (U[:, pu] * (sigma[:r].to(U.dtype) * sg)) @ V[:, pv].T
    if rms is not None:
        G = G * (rms / G.pow(2).mean().sqrt())
    return G.to(dtype)


def powerlaw_sigma(r: int, device) -> torch.Tensor:
    """sigma_i = 1 / i."""
    return 1.0 / torch.arange(1, r + 1, device=device, dtype=torch.float64)


def logspaced_sigma(r: int, decades: float, device) -> torch.Tensor:
    """sigma_i log-spaced from 1 down to 10^-decades."""
    return 10.0 ** (-decades * torch.arange(r, device=device, dtype=torch.float64) / max(r - 1, 1))


class TemplateBank:
    """A few Haar bases per dimension, reused across blocks (per-block permutation and signs
    make the blocks distinct) so that a 1B-model batch is generated in seconds."""

    def __init__(self, device, per_dim: int = 8, dtype=torch.float32, qr_on_host: bool = False):
        self.device, self.per_dim, self.dtype, self.qr_on_host = device, per_dim, dtype, qr_on_host
        self._bank = {}

    def get(self, n: int, idx: int) -> torch.Tensor:
        k = (n, idx % self.per_dim)
        if k not in self._bank:
            self._bank[k] = haar(n, self.device, idx % self.per_dim, dtype=self.dtype, qr_on_host=self.qr_on_host)
        return self._bank[k]


def powerlaw_blocks(shapes: Sequence[Tuple[int, int]], device, cfg: int = 3, rms: float = 0.01,
                    dtype=torch.bfloat16, bank: TemplateBank | None = None) -> List[torch.Tensor]:
    """One gradient block per shape with singular values proportional to 1 / i."""
    bank = bank or TemplateBank(device)
    out = []
    for b, (m, n) in enumerate(shapes):
        U, V = bank.get(m, b), bank.get(n, b + 3)
        out.append(spectrum_block(U, V, powerlaw_sigma(min(m, n), device), device, cfg, b, rms=rms, dtype=dtype))
    return out


def soap_gradient(U: torch.Tensor, V: torch.Tensor, step: int, device, *key: int, jitter: float = 0.3,
                  noise_frac: float = 0.1, rms: float = 0.01, dtype=torch.bfloat16) -> torch.Tensor:
    """Per-step gradient sharing the block's singular bases: sigma_i = (1/i)(1 + jitter u_i),
    u_i ~ U(-1, 1), plus dense Gaussian noise carrying `noise_frac` of the Frobenius norm."""
    m, n = U.shape[0], V.shape[0]
    r = min(m, n)
    g = _gen(device, 4, m, n, step, *key)
    u = torch.rand(r, generator=g, device=device, dtype=torch.float64) * 2 - 1
    sigma = powerlaw_sigma(r, device) * (1 + jitter * u)
    G = (U[:, :r] * sigma.to(U.dtype)) @ V[:, :r].T
    E = torch.randn(m, n, generator=g, device=device, dtype=U.dtype)
    G = G + E * (noise_frac * torch.linalg.norm(G) / torch.linalg.norm(E))
    G = G * (rms / G.pow(2).mean().sqrt())
    return G.to(dtype)
