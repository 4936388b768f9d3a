"""Seeded synthetic inputs for the gated subspace linear layer.

This module only *makes data*: weights, orthonormal bases and decode-token
activations with a prescribed residual ratio.  It holds none of the method's
arithmetic (no projection of a token onto a stored basis, no gate, no image
build), imports neither the HIP binding nor the CPU oracle, and is the one
module both sides may share.

Recipe (stands in for the trained GPT-2 / GPT-J / OPT weights and the
512-token calibration text of the paper's Section 6, none of which are needed
to exercise the kernel path):

* ``W``  : entries N(0, 1/d_in), stored fp32 or rounded to bf16 (RNE).
* ``U``  : Q factor of a seeded Gaussian d x k matrix, sign-fixed so that
           diag(R) > 0, generated in fp64 and then stored fp32 / bf16.
* ``x_t``: ``U a_t + sigma_t n_t`` with ``a_t ~ N(0, diag(i^-p))``, ``n_t`` a
           unit vector orthogonal to span(U) and ``sigma_t`` chosen so that the
           residual ratio of the paper's Eq. (rho) equals a prescribed
           ``rho*_t`` for the fp64 basis: ``sigma = rho* |a| / sqrt(1-rho*^2)``.
           Non-fired tokens get ``rho* = eps (0.2 + 0.6 u)``, fired tokens
           ``rho* = eps (1.2 + 3 u)``, ``u ~ U(0,1)``, so every designed ratio is
           at least 20 % away from the threshold.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 260503109

F32 = "f32"
BF16 = "bf16"


# ----------------------------------------------------------------------------
# storage formats
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) >> 16
    return u.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp32."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def store(a64: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp64 array to its storage dtype: fp32 array or uint16 bf16 bits."""
    if dtype == F32:
        return np.ascontiguousarray(a64, dtype=np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(np.asarray(a64, dtype=np.float32))
    raise ValueError(f"unknown storage dtype {dtype!r}")


def stored_to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact fp64 value of a stored array (for generator-side bookkeeping only)."""
    if dtype == F32:
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == BF16:
        return bf16_bits_to_f32(a).astype(np.float64)
    raise ValueError(f"unknown storage dtype {dtype!r}")


# ----------------------------------------------------------------------------
# operands
# ----------------------------------------------------------------------------
def make_weight(m: int, d: int, seed: int, dtype: str) -> np.ndarray:
    """W[m, d] row-major, entries N(0, 1/d), stored in ``dtype``."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((m, d), dtype=np.float32) * np.float32(1.0 / np.sqrt(d))
    return store(w, dtype)


def make_basis64(d: int, k: int, seed: int) -> np.ndarray:
    """Orthonormal U[d, k] in fp64: Q of a seeded Gaussian, columns sign-fixed."""
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((d, k))
    q, r = np.linalg.qr(g)
    s = np.sign(np.diag(r))
    s[s == 0] = 1.0
    return np.ascontiguousarray(q * s[None, :])


def choose_fired(T: int, n_fired: int, seed: int) -> np.ndarray:
    """Boolean[T] with exactly ``n_fired`` seeded positions set."""
    rng = np.random.default_rng(seed)
    mask = np.zeros(T, dtype=bool)
    if n_fired > 0:
        mask[rng.choice(T, size=n_fired, replace=False)] = True
    return mask


def bernoulli_fired(T: int, p: float, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.random(T) < p


def make_tokens64(
    U64: np.ndarray, fired: np.ndarray, eps: float, p: float, seed: int
) -> Tuple[np.ndarray, np.ndarray]:
    """Tokens X[T, d] (fp64) with designed residual ratios; returns (X, rho_star).

    ``U64`` must have orthonormal columns.  With k == d no orthogonal complement
    exists; then sigma is forced to 0 (rho* = 0) whatever ``fired`` says.
    """
    d, k = U64.shape
    T = int(fired.shape[0])
    rng = np.random.default_rng(seed)
    lam = np.arange(1, k + 1, dtype=np.float64) ** (-p)
    A = rng.standard_normal((T, k)) * np.sqrt(lam)[None, :]
    u = rng.random(T)
    rho_star = np.where(fired, eps * (1.2 + 3.0 * u), eps * (0.2 + 0.6 * u))
    G = rng.standard_normal((T, d))
    if k >= d:
        N = np.zeros((T, d))
        rho_star = np.zeros(T)
    else:
        # remove the span(U) component twice (second pass cleans rounding), then normalise
        for _ in range(2):
            G = G - (G @ U64) @ U64.T
        N = G / np.linalg.norm(G, axis=1, keepdims=True)
    anorm = np.linalg.norm(A, axis=1)
    sigma = rho_star * anorm / np.sqrt(1.0 - rho_star**2)
    X = A @ U64.T + sigma[:, None] * N
    return np.ascontiguousarray(X), rho_star


# ----------------------------------------------------------------------------
# workloads: input groups (one basis + one activation source) and their maps
# ----------------------------------------------------------------------------
@dataclass
class Group:
    """One distinct linear-layer input: basis U, tokens X and the maps that read it."""

    name: str
    d: int
    k: int
    U: np.ndarray            # stored dtype (fp32 array or uint16 bf16 bits), [d, k]
    X: np.ndarray            # stored dtype, [T, d]
    fired_design: np.ndarray  # bool[T], the designed gate outcome
    rho_star: np.ndarray      # designed residual ratio w.r.t. the fp64 basis
    maps: List[Tuple[str, int, np.ndarray]] = field(default_factory=list)  # (name, m, W[m,d])


@dataclass
class Workload:
    name: str
    wdtype: str
    xdtype: str
    eps: float
    T: int
    groups: List[Group]

    @property
    def dense_weight_bytes(self) -> int:
        b = 2 if self.wdtype == BF16 else 4
        return sum(m * g.d * b for g in self.groups for (_, m, _) in g.maps)

    @property
    def image_bytes(self) -> int:
        b = 2 if self.wdtype == BF16 else 4
        return sum(m * g.k * b for g in self.groups for (_, m, _) in g.maps)

    @property
    def basis_bytes(self) -> int:
        b = 2 if self.wdtype == BF16 else 4
        return sum(g.d * g.k * b for g in self.groups)


def _group(
    name: str,
    d: int,
    k: int,
    maps: Sequence[Tuple[str, int]],
    T: int,
    fired: np.ndarray,
    eps: float,
    p: float,
    seed: int,
    wdtype: str,
    xdtype: str,
    U64: Optional[np.ndarray] = None,
) -> Group:
    if U64 is None:
        U64 = make_basis64(d, k, seed + 1)
    X64, rho_star = make_tokens64(U64, fired, eps, p, seed + 2)
    g = Group(
        name=name,
        d=d,
        k=k,
        U=store(U64, wdtype),
        X=store(X64, xdtype),
        fired_design=fired.copy(),
        rho_star=rho_star,
    )
    for j, (mname, m) in enumerate(maps):
        g.maps.append((mname, m, make_weight(m, d, seed + 10 + j, wdtype)))
    return g


def gpt2_mlp_up(T: int = 16, n_fired: int = 4, seed: int = BASE_SEED) -> Workload:
    """GPT-2-small MLP up-projection, fp32: W 3072x768, k = 64, eps = 0.05."""
    eps = 0.05
    fired = choose_fired(T, n_fired, seed)
    g = _group("fc_in", 768, 64, [("fc_in", 3072)], T, fired, eps, 1.5, seed, F32, F32)
    return Workload("gpt2_mlp_up_f32", F32, F32, eps, T, [g])


def transformer_block(
    name: str,
    d: int,
    ffn: int,
    k: int,
    T: int,
    fire_rate: float,
    p: float,
    seed: int,
    eps: float = 0.05,
    wdtype: str = BF16,
    xdtype: str = F32,
    bernoulli: bool = False,
) -> Workload:
    """One transformer block's six linear maps over four distinct inputs.

    Inputs: the attention input (read by q, k, v), the attention output (read
    by o), the MLP input (fc_in) and the MLP hidden state (fc_out, d_in = ffn).
    Each input gets its own basis and its own seeded set of fired tokens.
    """
    specs = [
        ("attn_in", d, [("q", d), ("k", d), ("v", d)]),
        ("attn_out", d, [("o", d)]),
        ("mlp_in", d, [("fc_in", ffn)]),
        ("mlp_hidden", ffn, [("fc_out", d)]),
    ]
    groups = []
    for gi, (gname, din, maps) in enumerate(specs):
        gseed = seed + 100 * (gi + 1)
        if bernoulli:
            fired = bernoulli_fired(T, fire_rate, gseed)
        else:
            fired = choose_fired(T, int(round(fire_rate * T)), gseed)
        groups.append(_group(gname, din, min(k, din), maps, T, fired, eps, p, gseed, wdtype, xdtype))
    return Workload(name, wdtype, xdtype, eps, T, groups)


def gptj_block(T: int = 256, k: int = 256, fire_rate: float = 0.10, seed: int = BASE_SEED + 1000) -> Workload:
    """GPT-J-6B-shaped block at batch-1 decode: d = 4096, FFN = 16384, bf16 weights."""
    return transformer_block("gptj_block_bf16", 4096, 16384, k, T, fire_rate, 1.5, seed)


def opt_layer(layer: int, T: int, k: int, fire_rate: float, seed: int = BASE_SEED + 2000) -> Workload:
    """One OPT-6.7B-shaped layer (d = 4096, FFN = 16384), activation spectrum i^-1.2."""
    return transformer_block(
        f"opt_layer{layer}_k{k}_bf16", 4096, 16384, k, T, fire_rate, 1.2, seed + 7919 * layer
    )


def ffn_pair(T: int, k: int = 256, p_fire: float = 0.15, seed: int = BASE_SEED + 3000) -> Workload:
    """GPT-J-shaped fc_in / fc_out with a per-token Bernoulli(p_fire) gate design."""
    eps = 0.05
    groups = []
    for gi, (gname, din, m) in enumerate([("mlp_in", 4096, 16384), ("mlp_hidden", 16384, 4096)]):
        gseed = seed + 100 * (gi + 1)
        fired = bernoulli_fired(T, p_fire, gseed)
        groups.append(
            _group(gname, din, k, [("fc_in" if gi == 0 else "fc_out", m)], T, fired, eps, 1.5, gseed, BF16, F32)
        )
    return Workload("ffn_pair_bf16", BF16, F32, eps, T, groups)


def tiny(
    d: int, k: int, m: int, T: int, n_fired: int, seed: int, wdtype: str = F32, xdtype: str = F32, eps: float = 0.05
) -> Workload:
    """Small single-map workload of arbitrary (possibly odd) shape for brute-force checks."""
    fired = choose_fired(T, n_fired, seed)
    g = _group("g", d, k, [("w", m)], T, fired, eps, 1.5, seed, wdtype, xdtype)
    return Workload(f"tiny_{d}x{k}x{m}", wdtype, xdtype, eps, T, [g])
