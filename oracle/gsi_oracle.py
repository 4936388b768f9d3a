"""CPU oracle for the gated subspace linear layer -- TEST INFRASTRUCTURE ONLY.

A plain fp64 NumPy implementation of what the hot path computes, written from
the paper (Section 3: Eq. (decompose), Eq. (exact), Eq. (gate), Eq. (speedup),
Theorem "Per-layer error bound"; Section 4: Algorithm 1, "Storage"; Section 6:
Definition "Effective parameter count").  It is slow on purpose: every step is
one line of textbook linear algebra in the paper's order, with no blocking,
fusion or reordering, so it can be checked against the paper by eye.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this file.  It shares no code with the HIP path and imports nothing from it.

Notation: ``U`` is the paper's basis V_k (d x k), ``c`` its g = V_k^T x,
``M = W U`` the cached image, ``r`` the residual, ``rho`` the residual ratio.
Layouts are row-major: W[m, d], U[d, k], M[m, k], X[B, d], C[B, k], R[B, d],
Y[B, m].  Stored operands arrive as fp32 arrays or as uint16 bfloat16 bit
patterns and are widened exactly; all arithmetic after that is IEEE fp64.

Readings where the paper is silent or at odds with itself (each also listed in
the design notes):
  * tie: a token is on the fast path iff rho < eps (Definition "Activation basis
    and residual ratio", Algorithm 1), so the gate *fires* iff rho >= eps;
  * x = 0: rho is taken as 0 and the gate does not fire;
  * the norm is the Euclidean norm;
  * the fired-token output is M c + W r (Eq. (exact)); Algorithm 1 prints W x
    for the slow path, which is the same value in exact arithmetic --
    ``gated_linear_alg1`` is that variant;
  * eps is the fp32 value the device receives, widened to fp64;
  * the FP8 image of Section 7 "Combination with quantization" is OCP E4M3 with one
    power-of-two scale per output row (the paper names neither format nor scaling);
  * the residual norm of Eq. (rho) may be evaluated without forming r: for c = U^T x and ANY stored U,
    |x - U c|^2 = |x|^2 - |c|^2 + c^T (U^T U - I) c (``residual_norm_single_pass``) -- the same
    quantity, not an approximation; dropping the last term would assume U^T U = I exactly;
  * online basis maintenance (Section 5.3 "The cascade initialization", Section 5.4 "Time-dimension
    tracking", Section 7 "Online basis adaptation") names DGKS rank-1 updates without thresholds,
    capacity or eviction.  Reading: a basis lives in an array U[d, K] of fixed capacity K whose columns
    from k on are zero (a zero column changes neither c, r nor y); a token whose residual ratio is at
    least tau extends the basis, while k < K, by the normalised residual after classical Gram-Schmidt
    with one re-orthogonalisation pass ("twice is enough"); the new column is rounded to the basis'
    storage type and the image gains the column W u_new computed from that STORED column, so that
    M = W U keeps holding for the stored operands; nothing is ever evicted.

Every function here is pinned by tests that do not call the oracle to obtain
their expected value (hand-worked numbers, closed forms, invariants, brute
force on tiny inputs, values printed in the paper's tables).
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np

F32 = "f32"
BF16 = "bf16"


def widen(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact fp64 value of a stored operand (fp32 array, or uint16 bf16 bit patterns)."""
    if dtype == F32:
        a = np.asarray(a)
        if a.dtype != np.float32:
            raise TypeError("f32 operand must be a float32 array")
        return a.astype(np.float64)
    if dtype == BF16:
        a = np.asarray(a)
        if a.dtype != np.uint16:
            raise TypeError("bf16 operand must be a uint16 array of bit patterns")
        # bfloat16 is the upper half of an IEEE binary32 word
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


# ----------------------------------------------------------------------------
# Algorithm 1, lines 1-3 / Eq. (decompose), Eq. (gate)
# ----------------------------------------------------------------------------
def project(U: np.ndarray, X: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """c_t = U^T x_t ; r_t = x_t - U c_t ; |r_t| ; |x_t|, for every row t of X.

    U[d, k], X[B, d] in fp64.  Returns C[B, k], R[B, d], rnorm[B], xnorm[B].
    The residual is formed explicitly (Algorithm 1, line 2), never through
    |x|^2 - |c|^2.
    """
    U = np.asarray(U, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    B, d = X.shape
    k = U.shape[1]
    assert U.shape[0] == d
    C = np.empty((B, k))
    R = np.empty((B, d))
    rnorm = np.empty(B)
    xnorm = np.empty(B)
    for t in range(B):
        x = X[t]
        c = U.T @ x                      # Algorithm 1, line 1
        r = x - U @ c                    # Algorithm 1, line 2
        C[t] = c
        R[t] = r
        rnorm[t] = np.sqrt(np.sum(r * r))
        xnorm[t] = np.sqrt(np.sum(x * x))
    return C, R, rnorm, xnorm


def residual_ratio(rnorm: np.ndarray, xnorm: np.ndarray) -> np.ndarray:
    """rho_t = |r_t| / |x_t| (Eq. (gate)); 0 where x_t = 0."""
    rnorm = np.asarray(rnorm, dtype=np.float64)
    xnorm = np.asarray(xnorm, dtype=np.float64)
    rho = np.zeros_like(rnorm)
    nz = xnorm > 0
    rho[nz] = rnorm[nz] / xnorm[nz]
    return rho


def gate(rnorm: np.ndarray, xnorm: np.ndarray, eps: float) -> Tuple[np.ndarray, np.ndarray, int]:
    """Gate of Section 3.2: fired_t = (rho_t >= eps).  eps is rounded to fp32 first.

    Returns mask[B] (uint8), the ascending list of fired token indices (int32)
    and its length.
    """
    eps64 = float(np.float32(eps))
    rho = residual_ratio(rnorm, xnorm)
    fired = (np.asarray(xnorm) > 0) & (rho >= eps64)
    idx = np.nonzero(fired)[0].astype(np.int32)
    return fired.astype(np.uint8), idx, int(idx.shape[0])


# ----------------------------------------------------------------------------
# Eq. (rho) evaluated in one pass over the basis
# ----------------------------------------------------------------------------
def gram_defect(U: np.ndarray) -> np.ndarray:
    """E = U^T U - I for a stored basis U[d, k] (zero for an exactly orthonormal one)."""
    U = np.asarray(U, dtype=np.float64)
    return U.T @ U - np.eye(U.shape[1])


def residual_norm_single_pass(x: np.ndarray, c: np.ndarray, E: np.ndarray) -> float:
    """|x - U c| for c = U^T x without touching U again: sqrt(|x|^2 - |c|^2 + c^T E c), E = U^T U - I.

    Expanding |x - U c|^2 = |x|^2 - 2 c^T (U^T x) + c^T U^T U c with U^T x = c gives the formula for
    any U, orthonormal or not.  Negative round-off under the root is clamped to zero.
    """
    x = np.asarray(x, dtype=np.float64)
    c = np.asarray(c, dtype=np.float64)
    q = np.sum(x * x) - np.sum(c * c) + c @ (np.asarray(E, dtype=np.float64) @ c)
    return float(np.sqrt(max(q, 0.0)))


def project_single_pass(U: np.ndarray, E: np.ndarray, X: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """C[B, k], rnorm[B], xnorm[B] of Algorithm 1 lines 1 and 3 with the residual norm from the cached E."""
    U = np.asarray(U, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    C = np.empty((X.shape[0], U.shape[1]))
    rnorm = np.empty(X.shape[0])
    xnorm = np.empty(X.shape[0])
    for t in range(X.shape[0]):
        C[t] = U.T @ X[t]
        rnorm[t] = residual_norm_single_pass(X[t], C[t], E)
        xnorm[t] = np.sqrt(np.sum(X[t] * X[t]))
    return C, rnorm, xnorm


# ----------------------------------------------------------------------------
# Eq. (exact): cached image and the two paths
# ----------------------------------------------------------------------------
def build_image(W: np.ndarray, U: np.ndarray) -> np.ndarray:
    """M = W U (Eq. (exact)), fp64, not rounded.  W[m, d], U[d, k] -> M[m, k]."""
    return np.asarray(W, dtype=np.float64) @ np.asarray(U, dtype=np.float64)


def dense_linear(W: np.ndarray, X: np.ndarray) -> np.ndarray:
    """Baseline y_t = W x_t for every token.  W[m, d], X[B, d] -> Y[B, m]."""
    W = np.asarray(W, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    Y = np.empty((X.shape[0], W.shape[0]))
    for t in range(X.shape[0]):
        Y[t] = W @ X[t]
    return Y


def gated_linear(W: np.ndarray, M: np.ndarray, C: np.ndarray, R: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """y_t = M c_t for every token, plus W r_t for fired tokens (Eq. (exact), gated)."""
    W = np.asarray(W, dtype=np.float64)
    M = np.asarray(M, dtype=np.float64)
    B = C.shape[0]
    Y = np.empty((B, W.shape[0]))
    for t in range(B):
        y = M @ C[t]                     # Algorithm 1, line 5
        if mask[t]:
            y = y + W @ R[t]             # Eq. (exact), second term
        Y[t] = y
    return Y


def gated_linear_alg1(W: np.ndarray, M: np.ndarray, C: np.ndarray, X: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Algorithm 1 as printed: y_t = W x_t on the slow path, M c_t on the fast path."""
    W = np.asarray(W, dtype=np.float64)
    M = np.asarray(M, dtype=np.float64)
    B = C.shape[0]
    Y = np.empty((B, W.shape[0]))
    for t in range(B):
        Y[t] = W @ X[t] if mask[t] else M @ C[t]
    return Y


# ----------------------------------------------------------------------------
# Section 7 "Combination with quantization": the cached image stored in 8-bit floating point
# ----------------------------------------------------------------------------
# The paper names FP8 and the 2x smaller fast-path read, not a format.  Reading taken here: the OCP 8-bit
# E4M3 encoding (sign, 4 exponent bits with bias 7, 3 mantissa bits; exponent field 0 is subnormal,
# m/8 * 2^-6; exponent field 15 with mantissa 7 is NaN, there are no infinities; largest finite value
# 1.75 * 2^8 = 448), one power-of-two scale per output row, round to nearest with ties to the even code.
FP8_MAX = 448.0


def fp8_e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """Value of every E4M3 code (uint8 -> fp64), NaN for the two NaN codes."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 0x7).astype(np.float64)
    val = np.where(e == 0, (m / 8.0) * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    val = np.where((e == 15) & ((c & 0x7) == 7), np.nan, val)
    return sign * val


def fp8_e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of every element (ties to the even code), |x| above 448 saturating to 448.

    Works on the value grid itself: in the binade 2^e <= |x| < 2^(e+1) (e clamped to the subnormal
    exponent -6 below) the codes are spaced 2^(e-3) apart, so the code index is |x| / 2^(e-3) rounded
    half-to-even; an index that rounds up to 16 is the first code of the next binade.
    """
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    out = np.zeros(x.shape, dtype=np.uint8)
    nan = np.isnan(x)
    a = np.where(nan, 0.0, np.minimum(a, FP8_MAX))
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0))).astype(np.int64)
    # log2 of a value just below a power of two may round up: correct by comparison
    e = np.where(np.exp2(e.astype(np.float64)) > a, e - 1, e)
    e = np.where(np.exp2((e + 1).astype(np.float64)) <= a, e + 1, e)
    e = np.maximum(e, -6)
    step = np.exp2((e - 3).astype(np.float64))
    q = np.rint(a / step).astype(np.int64)        # numpy rounds half to even; a / step is exact
    # q counts steps from zero of this binade's grid: normal binades have q in [8, 16], the
    # subnormal one q in [0, 8]
    carry = q == 16
    e = np.where(carry, e + 1, e)
    q = np.where(carry, 8, q)
    normal = q >= 8
    field = np.where(normal, e + 7, 0)
    mant = np.where(normal, q - 8, q)
    code = (field << 3) | mant
    code = np.where(a > 0, code, 0)
    code = np.where(np.signbit(x) & ~nan, code | 0x80, code)
    out[...] = np.where(nan, 0x7F, code).astype(np.uint8)
    return out


def fp8_row_scale(M: np.ndarray) -> np.ndarray:
    """Per-row power-of-two scale: the smallest 2^e (e in [-126, 127]) with max_j |M_ij| / 2^e <= 448; 1 for a zero row.

    Elements that are not finite take no part in the choice (they saturate, or stay NaN, when encoded).
    """
    M = np.asarray(M, dtype=np.float64)
    mag = np.where(np.isfinite(M), np.abs(M), 0.0)
    amax = np.max(mag, axis=1) if M.shape[1] else np.zeros(M.shape[0])
    scale = np.ones(M.shape[0])
    for i, a in enumerate(amax):
        if a > 0:
            e = int(np.ceil(np.log2(a / FP8_MAX)))
            while a / 2.0 ** e > FP8_MAX:       # guard the rounding of log2
                e += 1
            while a / 2.0 ** (e - 1) <= FP8_MAX:
                e -= 1
            scale[i] = 2.0 ** min(max(e, -126), 127)
    return scale


def quantize_image_fp8(M: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """codes[m, k] (uint8), scale[m]: codes_ij = E4M3(M_ij / scale_i).  M is the stored image, widened."""
    M = np.asarray(M, dtype=np.float64)
    scale = fp8_row_scale(M)
    return fp8_e4m3_encode(M / scale[:, None]), scale


def dequantize_image_fp8(codes: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """M_ij = scale_i * value(codes_ij), fp64."""
    return fp8_e4m3_decode(codes) * np.asarray(scale, dtype=np.float64)[:, None]


# ----------------------------------------------------------------------------
# Sections 5.3, 5.4 and 7 "Online basis adaptation": rank-1 extension of the basis (DGKS)
# ----------------------------------------------------------------------------
def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to the storage type, to nearest with ties to even; returns what ``widen`` reads."""
    a = np.asarray(a, dtype=np.float64)
    f = a.astype(np.float32)
    if dtype == F32:
        return f
    if dtype == BF16:
        # fp64 -> bf16 in one rounding: a lies between the truncation of its fp32 value and the next bf16
        # (if the fp32 rounding carried up to a bf16 value, that value is the truncation and it is nearest)
        bits = f.view(np.uint32)
        lo = bits & np.uint32(0xFFFF0000)                     # truncated toward zero in magnitude
        hi = lo + np.uint32(0x10000)                          # next bf16 away from zero
        vlo = lo.view(np.float32).astype(np.float64)
        vhi = hi.view(np.float32).astype(np.float64)
        dlo, dhi = np.abs(a - vlo), np.abs(vhi - a)
        up = (dhi < dlo) | ((dhi == dlo) & (((lo >> np.uint32(16)) & np.uint32(1)) == 1))
        out = np.where(up, hi, lo)
        return (out >> np.uint32(16)).astype(np.uint16)
    raise ValueError(f"unknown dtype {dtype!r}")


def dgks_direction(U: np.ndarray, x: np.ndarray) -> Tuple[np.ndarray, float, float]:
    """The unit vector that extends span(U) to contain x, and the residual norms of the two passes.

    Classical Gram-Schmidt against the columns of U followed by one re-orthogonalisation pass:
      c = U^T x, r = x - U c;   s = U^T r, r2 = r - U s;   u_new = r2 / |r2|.
    Returns (u_new, |r|, |r2|); u_new is zero when r2 vanishes (x already in the span).
    """
    U = np.asarray(U, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    c = U.T @ x
    r = x - U @ c
    s = U.T @ r
    r2 = r - U @ s
    n1 = float(np.sqrt(np.sum(r * r)))
    n2 = float(np.sqrt(np.sum(r2 * r2)))
    u = r2 / n2 if n2 > 0 else np.zeros_like(r2)
    return u, n1, n2


def extend_basis(U_store: np.ndarray, udtype: str, k: int, x: np.ndarray, tau: float) -> Tuple[np.ndarray, int, bool]:
    """One step of the tracker on a basis array of fixed capacity.

    ``U_store[d, K]`` holds the stored basis (fp32, or bf16 bit patterns) with columns k..K-1 zero.  The token x
    extends it iff x != 0, |x - U U^T x| / |x| >= tau (tau rounded to fp32 like eps) and k < K; the new column is
    the DGKS direction rounded to the storage type.  Returns (new array, new k, extended?).
    """
    U = widen(U_store, udtype)
    x = np.asarray(x, dtype=np.float64)
    u, n1, n2 = dgks_direction(U, x)
    xn = float(np.sqrt(np.sum(x * x)))
    K = U.shape[1]
    if not (xn > 0 and n1 / xn >= float(np.float32(tau)) and k < K and n2 > 0):
        return U_store, k, False
    out = np.array(U_store, copy=True)
    out[:, k] = round_to_storage(u, udtype)
    return out, k + 1, True


def extend_image(M: np.ndarray, k: int, W: np.ndarray, u_stored: np.ndarray) -> np.ndarray:
    """The matching append M <- [M, W u_new] into column k of M[m, K], fp64, not rounded; u_stored is the
    widened STORED new column, so that M = W U holds for the stored basis (Eq. (exact))."""
    out = np.array(np.asarray(M, dtype=np.float64), copy=True)
    out[:, k] = np.asarray(W, dtype=np.float64) @ np.asarray(u_stored, dtype=np.float64)
    return out


def track_basis(U_store: np.ndarray, udtype: str, k: int, X: np.ndarray, tau: float) -> Tuple[np.ndarray, int, List[int]]:
    """Section 5.4: every token in turn is tested against the current basis and may extend it.

    Returns the final array, the final rank and the list of tokens that extended the basis.  Section 5.3's
    cascade is this function started from the previous layer's basis instead of from an empty one.
    """
    grew = []
    for t in range(np.asarray(X).shape[0]):
        U_store, k, ext = extend_basis(U_store, udtype, k, X[t], tau)
        if ext:
            grew.append(t)
    return U_store, k, grew


# ----------------------------------------------------------------------------
# a chain of per-layer linear maps (Section 1: every map of a block shares the
# projection of its input)
# ----------------------------------------------------------------------------
def prepare_stack(groups: Sequence[dict]) -> List[dict]:
    """Widen stored operands and build the fp64 images once (the one-time set-up of Section 4).

    ``groups``: list of dicts {U, udtype, maps: [(name, W, wdtype), ...]}.
    """
    out = []
    for g in groups:
        U = widen(g["U"], g["udtype"])
        maps = []
        for name, W, wdtype in g["maps"]:
            W64 = widen(W, wdtype)
            maps.append((name, W64, build_image(W64, U)))
        out.append({"U": U, "maps": maps})
    return out


def run_stack(prepared: Sequence[dict], Xs: Sequence[np.ndarray], eps: float) -> List[dict]:
    """One pass: per input group project + gate once, then one gated linear map per weight.

    ``Xs[g]`` is the fp64 token block X[B, d_g] of group g.  Returns per group
    {C, R, rnorm, xnorm, rho, mask, fired_idx, n_fired, Y: {name: Y[B, m]}}.
    """
    res = []
    for g, X in zip(prepared, Xs):
        C, R, rn, xn = project(g["U"], X)
        mask, idx, n = gate(rn, xn, eps)
        Y = {name: gated_linear(W64, M64, C, R, mask) for name, W64, M64 in g["maps"]}
        res.append(
            {"C": C, "R": R, "rnorm": rn, "xnorm": xn, "rho": residual_ratio(rn, xn),
             "mask": mask, "fired_idx": idx, "n_fired": n, "Y": Y}
        )
    return res


def run_dense_stack(prepared: Sequence[dict], Xs: Sequence[np.ndarray]) -> List[Dict[str, np.ndarray]]:
    """The baseline the method is compared with: y = W x for every map and token."""
    return [{name: dense_linear(W64, X) for name, W64, _ in g["maps"]} for g, X in zip(prepared, Xs)]


# ----------------------------------------------------------------------------
# closed forms used for reporting
# ----------------------------------------------------------------------------
def effective_speedup(f: float, d: int, k: int) -> float:
    """Eq. (speedup): S = 1 / (f / (d/k) + (1 - f)) for fast-path fraction f."""
    return 1.0 / (f / (d / k) + (1.0 - f))


def model_speedup(layers: Sequence[Tuple[float, int, int, float]]) -> float:
    """Model-wide speedup: harmonic mean of S_l weighted by weight-read volume (Section 3.2).

    ``layers``: (f_l, d_l, k_l, volume_l).  Equals total dense volume over total gated volume.
    """
    vol = sum(v for _, _, _, v in layers)
    return vol / sum(v / effective_speedup(f, d, k) for f, d, k, v in layers)


def effective_params(layers: Sequence[Tuple[int, int, int, int, float]]) -> float:
    """Definition "Effective parameter count": sum_l N_W d_out [f k + (1 - f) d].

    ``layers``: (N_W, d_out, d, k, f) per layer.
    """
    return float(sum(n * dout * (f * k + (1.0 - f) * d) for n, dout, d, k, f in layers))


def image_storage_elems(n_maps_dout: Sequence[int], L: int, k: int) -> int:
    """Section 4 "Storage": elements of cached images = L * k * sum of d_out over the maps."""
    return L * k * int(sum(n_maps_dout))


def basis_storage_elems(L: int, d: int, k: int) -> int:
    """Section 4 "Storage": elements of the per-layer bases = L d k."""
    return L * d * k


def error_bound(W: np.ndarray, eps: float, xnorm: np.ndarray) -> np.ndarray:
    """Theorem "Per-layer error bound": |W r| <= |W|_2 eps |x| on the fast path."""
    s = np.linalg.svd(np.asarray(W, dtype=np.float64), compute_uv=False)[0]
    return s * float(np.float32(eps)) * np.asarray(xnorm, dtype=np.float64)
