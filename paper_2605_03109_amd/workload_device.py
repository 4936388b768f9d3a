"""Seeded synthetic inputs generated on the GPU, for workloads too large to make with NumPy in reasonable time
(the 32-layer stack, ragged decode batches, the prefill-sized batch).

Same recipe as ``workload.py`` (which see), written with torch tensor ops in fp64 on the device.  Like that
module it only *makes data* -- weights, orthonormal bases, tokens with a prescribed residual ratio -- and
holds none of the method's arithmetic.  The random streams differ from the NumPy generator's, so a workload
made here is not bit-identical to one of the same name made there; each is reproducible from its seed.
"""
from __future__ import annotations

import math
from typing import Tuple

import torch

BASE_SEED = 260503109


def generator(seed: int, device: str = "cuda") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_weight(m: int, d: int, gen: torch.Generator) -> torch.Tensor:
    """W[m, d], entries N(0, 1/d), rounded to bf16 (RNE)."""
    w = torch.randn((m, d), generator=gen, device=gen.device, dtype=torch.float32)
    w.mul_(1.0 / math.sqrt(d))
    return w.to(torch.bfloat16)


def make_basis64(d: int, k: int, gen: torch.Generator, host_qr: bool = False) -> torch.Tensor:
    """Orthonormal U[d, k] in fp64: Q of a seeded Gaussian, columns sign-fixed.  A leading block U[:, :k']
    of the result is itself an orthonormal basis (nested bases across ranks)."""
    g = torch.randn((d, k), generator=gen, device=gen.device, dtype=torch.float64)
    try:
        if host_qr:
            raise RuntimeError("host factorisation asked for")
        q, r = torch.linalg.qr(g)
    except RuntimeError:  # no device QR in this build, or the caller wants the host's: factor on the host
        q, r = torch.linalg.qr(g.cpu())
        q, r = q.to(g.device), r.to(g.device)
    s = torch.sign(torch.diagonal(r))
    s[s == 0] = 1.0
    return (q * s[None, :]).contiguous()


def choose_fired(T: int, n_fired: int, gen: torch.Generator) -> torch.Tensor:
    """bool[T] with exactly ``n_fired`` seeded positions set."""
    mask = torch.zeros(T, dtype=torch.bool, device=gen.device)
    if n_fired > 0:
        perm = torch.randperm(T, generator=gen, device=gen.device)
        mask[perm[:n_fired]] = True
    return mask


def bernoulli_fired(T: int, p: float, gen: torch.Generator) -> torch.Tensor:
    return torch.rand(T, generator=gen, device=gen.device, dtype=torch.float64) < p


def make_tokens(U64: torch.Tensor, fired: torch.Tensor, eps: float, p: float, gen: torch.Generator,
                chunk: int = 4096) -> Tuple[torch.Tensor, torch.Tensor]:
    """Tokens X[T, d] (fp32) = U a + sigma n with residual ratio rho* w.r.t. the fp64 basis; returns (X, rho*).

    a ~ N(0, diag(i^-p)); n unit, orthogonal to span(U); sigma = rho* |a| / sqrt(1 - rho*^2);
    rho* = eps (1.2 + 3u) for fired tokens, eps (0.2 + 0.6u) otherwise."""
    d, k = U64.shape
    T = int(fired.shape[0])
    dev = U64.device
    lam = torch.arange(1, k + 1, device=dev, dtype=torch.float64) ** (-p)
    X = torch.empty((T, d), device=dev, dtype=torch.float32)
    rho = torch.empty(T, device=dev, dtype=torch.float64)
    for t0 in range(0, T, chunk):
        t1 = min(T, t0 + chunk)
        n = t1 - t0
        A = torch.randn((n, k), generator=gen, device=dev, dtype=torch.float64) * torch.sqrt(lam)[None, :]
        u = torch.rand(n, generator=gen, device=dev, dtype=torch.float64)
        f = fired[t0:t1]
        rs = torch.where(f, eps * (1.2 + 3.0 * u), eps * (0.2 + 0.6 * u))
        G = torch.randn((n, d), generator=gen, device=dev, dtype=torch.float64)
        if k >= d:
            N = torch.zeros_like(G)
            rs = torch.zeros_like(rs)
        else:
            for _ in range(2):  # the second pass cleans the rounding of the first
                G = G - (G @ U64) @ U64.T
            N = G / torch.linalg.norm(G, dim=1, keepdim=True)
        sigma = rs * torch.linalg.norm(A, dim=1) / torch.sqrt(1.0 - rs * rs)
        X[t0:t1] = (A @ U64.T + sigma[:, None] * N).to(torch.float32)
        rho[t0:t1] = rs
    return X, rho
