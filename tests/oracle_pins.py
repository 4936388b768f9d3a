"""Pins for the CPU oracle: each takes the oracle module ``O`` and asserts a fact that is fixed by
the paper or by mathematics, never by the oracle's own output.

They are written as functions of ``O`` so that the same pins can be run against deliberately
broken copies of the oracle (tests/test_oracle_mutants.py) to show that a plausible mistake in
any step is caught by at least one of them.
"""
import math

import numpy as np

from paper_2605_03109_amd import workload as wl


def _fsum_matvec(A, x):
    """Brute-force y = A x with exactly rounded sums (math.fsum), plain Python loops."""
    return np.array([math.fsum(float(A[i, j]) * float(x[j]) for j in range(A.shape[1])) for i in range(A.shape[0])])


def _fsum_matmul(A, B):
    return np.array(
        [[math.fsum(float(A[i, l]) * float(B[l, j]) for l in range(A.shape[1])) for j in range(B.shape[1])]
         for i in range(A.shape[0])]
    )


def pin_hand_worked_2d(O):
    # Worked by hand: U = (3/5, 4/5)^T, x = (1, 2), W = [[1,2],[3,4],[5,6]].
    # c = 11/5; U c = (33/25, 44/25); r = (-8/25, 6/25); |r| = 2/5; |x| = sqrt 5;
    # M = W U = (11/5, 5, 39/5); M c = (4.84, 11, 17.16); W r = (0.16, 0, -0.16); M c + W r = W x = (5, 11, 17).
    U = np.array([[0.6], [0.8]])
    X = np.array([[1.0, 2.0]])
    W = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    C, R, rn, xn = O.project(U, X)
    assert np.allclose(C, [[2.2]], rtol=0, atol=1e-15)
    assert np.allclose(R, [[-0.32, 0.24]], rtol=0, atol=1e-15)
    assert abs(rn[0] - 0.4) < 1e-15 and abs(xn[0] - math.sqrt(5.0)) < 1e-15
    assert abs(O.residual_ratio(rn, xn)[0] - 0.4 / math.sqrt(5.0)) < 1e-15
    M = O.build_image(W, U)
    assert M.shape == (3, 1) and np.allclose(M[:, 0], [2.2, 5.0, 7.8], rtol=0, atol=1e-14)
    y_fast = O.gated_linear(W, M, C, R, np.array([0], dtype=np.uint8))
    y_slow = O.gated_linear(W, M, C, R, np.array([1], dtype=np.uint8))
    assert np.allclose(y_fast, [[4.84, 11.0, 17.16]], rtol=0, atol=1e-13)
    assert np.allclose(y_slow, [[5.0, 11.0, 17.0]], rtol=0, atol=1e-13)
    y_alg1 = O.gated_linear_alg1(W, M, C, X, np.array([1], dtype=np.uint8))
    assert np.allclose(y_alg1, [[5.0, 11.0, 17.0]], rtol=0, atol=1e-13)
    assert np.allclose(O.dense_linear(W, X), [[5.0, 11.0, 17.0]], rtol=0, atol=1e-13)
    # rho = 0.1789 >= 0.05 fires; at eps = 0.2 it does not
    assert O.gate(rn, xn, 0.05)[2] == 1 and O.gate(rn, xn, 0.2)[2] == 0


def pin_axis_aligned_basis(O):
    # U = columns of the identity: c picks coordinates, r zeroes them, M picks columns of W.
    rng = np.random.default_rng(11)
    d, k, m, B = 9, 4, 5, 3
    sel = np.array([7, 2, 5, 0])
    U = np.zeros((d, k))
    U[sel, np.arange(k)] = 1.0
    X = rng.standard_normal((B, d))
    W = rng.standard_normal((m, d))
    C, R, rn, xn = O.project(U, X)
    assert np.array_equal(C, X[:, sel])
    Rexp = X.copy()
    Rexp[:, sel] = 0.0
    assert np.array_equal(R, Rexp)
    rest = np.setdiff1d(np.arange(d), sel)
    for t in range(B):
        assert abs(rn[t] - math.sqrt(math.fsum(v * v for v in X[t, rest]))) < 1e-14
        assert abs(xn[t] - math.sqrt(math.fsum(v * v for v in X[t]))) < 1e-14
    M = O.build_image(W, U)
    assert np.array_equal(M, W[:, sel])
    Y = O.gated_linear(W, M, C, R, np.array([1, 0, 1], dtype=np.uint8))
    for t, fired in enumerate([1, 0, 1]):
        cols = np.arange(d) if fired else sel
        yexp = _fsum_matvec(W[:, cols], X[t, cols])
        assert np.allclose(Y[t], yexp, rtol=0, atol=1e-13)


def pin_brute_force_tiny(O):
    # Odd, non-square shapes; exactly rounded loop sums as the reference.
    rng = np.random.default_rng(5)
    d, k, m, B = 12, 3, 5, 4
    U, _ = np.linalg.qr(rng.standard_normal((d, k)))
    X = rng.standard_normal((B, d))
    W = rng.standard_normal((m, d))
    C, R, rn, xn = O.project(U, X)
    for t in range(B):
        c = _fsum_matvec(U.T, X[t])
        assert np.allclose(C[t], c, rtol=0, atol=1e-14)
        uc = _fsum_matvec(U, c)
        assert np.allclose(R[t], X[t] - uc, rtol=0, atol=1e-14)
    M = O.build_image(W, U)
    assert np.allclose(M, _fsum_matmul(W, U), rtol=0, atol=1e-14)
    mask = np.array([1, 0, 0, 1], dtype=np.uint8)
    Y = O.gated_linear(W, M, C, R, mask)
    for t in range(B):
        y = _fsum_matvec(_fsum_matmul(W, U), _fsum_matvec(U.T, X[t]))
        if mask[t]:
            y = y + _fsum_matvec(W, X[t] - _fsum_matvec(U, _fsum_matvec(U.T, X[t])))
        assert np.allclose(Y[t], y, rtol=0, atol=1e-13)
    assert np.allclose(O.dense_linear(W, X), np.array([_fsum_matvec(W, X[t]) for t in range(B)]), rtol=0, atol=1e-13)


def pin_orthogonality_and_pythagoras(O):
    # r is orthogonal to span(U) and |x|^2 = |c|^2 + |r|^2 for an orthonormal basis.
    U = wl.make_basis64(96, 17, 3)
    assert np.max(np.abs(U.T @ U - np.eye(17))) < 1e-12
    X = np.random.default_rng(1).standard_normal((6, 96))
    C, R, rn, xn = O.project(U, X)
    assert np.max(np.abs(R @ U)) < 1e-12 * np.max(xn)
    assert np.allclose(xn**2, np.sum(C * C, axis=1) + rn**2, rtol=1e-12, atol=0)
    assert np.allclose(X, C @ U.T + R, rtol=0, atol=1e-13)
    rho = O.residual_ratio(rn, xn)
    assert np.all(rho >= 0) and np.all(rho <= 1.0 + 1e-15)


def pin_designed_rho(O):
    # The generator fixes rho_t in closed form: x = U a + sigma n, n unit and orthogonal to U
    # => rho = sigma / sqrt(|a|^2 + sigma^2) = rho*.  Also the designed fire count is hit exactly.
    w = wl.tiny(d=80, k=12, m=7, T=24, n_fired=7, seed=99)
    g = w.groups[0]
    U = O.widen(g.U, w.wdtype)
    X = O.widen(g.X, w.xdtype)
    C, R, rn, xn = O.project(U, X)
    rho = O.residual_ratio(rn, xn)
    assert np.allclose(rho, g.rho_star, rtol=0, atol=5e-7)  # fp32 storage of U and x
    mask, idx, n = O.gate(rn, xn, w.eps)
    assert n == 7 and np.array_equal(mask.astype(bool), g.fired_design)
    assert np.array_equal(idx, np.nonzero(g.fired_design)[0]) and idx.dtype == np.int32
    assert np.all(np.diff(idx) > 0)


def pin_full_rank_basis(O):
    # k = d: the projection is the identity, r = 0, rho = 0, M c = W x.
    rng = np.random.default_rng(2)
    d, m = 10, 6
    U = wl.make_basis64(d, d, 8)
    X = rng.standard_normal((3, d))
    W = rng.standard_normal((m, d))
    C, R, rn, xn = O.project(U, X)
    assert np.max(np.abs(R)) < 1e-14 and np.max(rn / xn) < 1e-14
    Y = O.gated_linear(W, O.build_image(W, U), C, R, np.zeros(3, dtype=np.uint8))
    assert np.allclose(Y, np.array([_fsum_matvec(W, x) for x in X]), rtol=0, atol=1e-13)


def pin_monotone_in_k(O):
    # Proposition "Monotonicity": nested bases => rho(k+1) <= rho(k); fired set shrinks.
    U = wl.make_basis64(64, 40, 21)
    X = np.random.default_rng(4).standard_normal((8, 64))
    prev = None
    prev_mask = None
    for k in (1, 2, 5, 8, 16, 32, 40):
        _, _, rn, xn = O.project(U[:, :k], X)
        rho = O.residual_ratio(rn, xn)
        mask = O.gate(rn, xn, 0.7)[0]
        if prev is not None:
            assert np.all(rho <= prev + 1e-15)
            assert np.all(mask <= prev_mask)
        prev, prev_mask = rho, mask


def pin_all_fire_is_dense(O):
    # Eq. (exact) is an identity: when every gate fires, y = W x.  Reference: extended-precision einsum.
    rng = np.random.default_rng(6)
    d, k, m, B = 70, 9, 33, 5
    U = wl.make_basis64(d, k, 1)
    X = rng.standard_normal((B, d))
    W = rng.standard_normal((m, d))
    C, R, rn, xn = O.project(U, X)
    mask, idx, n = O.gate(rn, xn, 0.0)
    assert n == B and np.all(mask == 1)
    M = O.build_image(W, U)
    Y = O.gated_linear(W, M, C, R, mask)
    Yd = np.einsum("ij,tj->ti", W.astype(np.longdouble), X.astype(np.longdouble)).astype(np.float64)
    assert np.max(np.linalg.norm(Y - Yd, axis=1) / np.linalg.norm(Yd, axis=1)) < 1e-13
    assert np.max(np.abs(O.gated_linear_alg1(W, M, C, X, mask) - Yd)) < 1e-12
    assert np.max(np.abs(O.dense_linear(W, X) - Yd)) < 1e-12


def pin_none_fire_is_static_projection(O):
    # eps > 1: no token fires and y = W (U (U^T x)) -- evaluated right-to-left here, so it never forms W U.
    rng = np.random.default_rng(7)
    d, k, m, B = 50, 6, 21, 4
    U = wl.make_basis64(d, k, 2)
    X = rng.standard_normal((B, d))
    W = rng.standard_normal((m, d))
    C, R, rn, xn = O.project(U, X)
    mask, idx, n = O.gate(rn, xn, 1.5)
    assert n == 0 and idx.shape == (0,) and not mask.any()
    Y = O.gated_linear(W, O.build_image(W, U), C, R, mask)
    for t in range(B):
        x = X[t].astype(np.longdouble)
        yexp = W.astype(np.longdouble) @ (U.astype(np.longdouble) @ (U.T.astype(np.longdouble) @ x))
        assert np.linalg.norm(Y[t] - yexp.astype(np.float64)) < 1e-13 * np.linalg.norm(yexp.astype(np.float64)) + 1e-14


def pin_error_bound(O):
    # Theorem "Per-layer error bound": non-fired => |W x - y| = |W r| <= |W|_2 eps |x|; fired => 0.
    w = wl.tiny(d=64, k=10, m=40, T=32, n_fired=9, seed=5)
    g = w.groups[0]
    U = O.widen(g.U, w.wdtype)
    X = O.widen(g.X, w.xdtype)
    W = O.widen(g.maps[0][2], w.wdtype)
    C, R, rn, xn = O.project(U, X)
    mask, _, _ = O.gate(rn, xn, w.eps)
    Y = O.gated_linear(W, O.build_image(W, U), C, R, mask)
    Yd = np.einsum("ij,tj->ti", W.astype(np.longdouble), X.astype(np.longdouble)).astype(np.float64)
    err = np.linalg.norm(Y - Yd, axis=1)
    # |W|_2 from power iteration on W^T W (independent of the oracle's SVD call)
    v = np.ones(W.shape[1])
    for _ in range(500):
        v = W.T @ (W @ v)
        v /= np.linalg.norm(v)
    s2 = np.linalg.norm(W @ v)
    bound = s2 * float(np.float32(w.eps)) * xn
    assert np.all(err[mask == 0] <= bound[mask == 0] * (1 + 1e-9))
    assert np.all(err[mask == 0] > 0)            # the fast path *is* an approximation
    assert np.all(err[mask == 1] <= 1e-12 * np.linalg.norm(Yd, axis=1)[mask == 1])
    assert np.allclose(O.error_bound(W, w.eps, xn), bound, rtol=1e-6)


def pin_gate_boundary(O):
    # fast path iff rho < eps; fires iff rho >= eps (Definition "Activation basis and residual ratio", Alg. 1).
    eps32 = np.float32(0.05)
    e = float(eps32)
    xn = np.array([1.0, 1.0, 1.0, 2.0, 0.0, 4.0, 1.0])
    rn = np.array([e, np.nextafter(e, 0.0), np.nextafter(e, 1.0), 2.0 * e, 0.0, 0.1, 0.0])
    mask, idx, n = O.gate(rn, xn, 0.05)
    assert mask.dtype == np.uint8 and mask.tolist() == [1, 0, 1, 1, 0, 0, 0]
    assert idx.tolist() == [0, 2, 3] and n == 3
    # eps = 0: every token with x != 0 fires, even with r = 0; x = 0 never fires
    mask0, idx0, n0 = O.gate(rn, xn, 0.0)
    assert mask0.tolist() == [1, 1, 1, 1, 0, 1, 1] and n0 == 6
    # eps > 1 can never fire since rho <= 1
    assert O.gate(np.array([1.0, 0.5]), np.array([1.0, 1.0]), 1.0000001)[2] == 0
    # the threshold is the fp32 value of eps, not the fp64 literal 0.05 (0.05f > 0.05)
    between = 0.5 * (0.05 + e)
    assert O.gate(np.array([between]), np.array([1.0]), 0.05)[2] == 0


def pin_batch_equals_per_token(O):
    rng = np.random.default_rng(12)
    d, k, m, B = 33, 5, 11, 6
    U = wl.make_basis64(d, k, 3)
    X = rng.standard_normal((B, d))
    W = rng.standard_normal((m, d))
    C, R, rn, xn = O.project(U, X)
    mask, _, _ = O.gate(rn, xn, 0.93)
    assert 0 < mask.sum() < B
    M = O.build_image(W, U)
    Y = O.gated_linear(W, M, C, R, mask)
    for t in range(B):
        Ct, Rt, rnt, xnt = O.project(U, X[t : t + 1])
        mt, _, _ = O.gate(rnt, xnt, 0.93)
        Yt = O.gated_linear(W, M, Ct, Rt, mt)
        assert np.array_equal(Ct[0], C[t]) and np.array_equal(Rt[0], R[t]) and mt[0] == mask[t]
        assert np.array_equal(Yt[0], Y[t])


def pin_widen(O):
    # bfloat16 bit patterns with known values: sign(1) exponent(8) mantissa(7)
    bits = np.array([0x3F80, 0xC000, 0x3FC0, 0x0000, 0x8000, 0x0001, 0x7F7F, 0x3DCD], dtype=np.uint16)
    vals = O.widen(bits, "bf16")
    exp = [1.0, -2.0, 1.5, 0.0, -0.0, 2.0**-133, (2.0 - 2.0**-7) * 2.0**127, 0.10009765625]
    assert vals.dtype == np.float64 and vals.tolist() == exp
    assert math.copysign(1.0, vals[4]) == -1.0
    a = np.array([0.1, -3.25], dtype=np.float32)
    assert O.widen(a, "f32").tolist() == [float(np.float32(0.1)), -3.25]


def pin_stack(O):
    # run_stack = project + gate once per input, one gated map per weight; dense stack = W x.
    w = wl.transformer_block("t", d=32, ffn=64, k=6, T=10, fire_rate=0.3, p=1.5, seed=77, wdtype="bf16")
    groups = [{"U": g.U, "udtype": w.wdtype, "maps": [(n, W, w.wdtype) for n, _, W in g.maps]} for g in w.groups]
    prep = O.prepare_stack(groups)
    Xs = [O.widen(g.X, w.xdtype) for g in w.groups]
    res = O.run_stack(prep, Xs, w.eps)
    dense = O.run_dense_stack(prep, Xs)
    assert [sorted(r["Y"]) for r in res] == [["k", "q", "v"], ["o"], ["fc_in"], ["fc_out"]]
    for g, r, dn, X in zip(w.groups, res, dense, Xs):
        assert r["n_fired"] == 3 and np.array_equal(r["mask"].astype(bool), g.fired_design)
        Ub = wl.bf16_bits_to_f32(g.U).astype(np.longdouble)
        for name, m, Wb in g.maps:
            Wl = wl.bf16_bits_to_f32(Wb).astype(np.longdouble)
            Yd = (X.astype(np.longdouble) @ Wl.T).astype(np.float64)
            assert np.allclose(dn[name], Yd, rtol=0, atol=1e-12)
            Ys = (((X.astype(np.longdouble) @ Ub) @ Ub.T) @ Wl.T).astype(np.float64)
            fired = g.fired_design
            assert np.allclose(r["Y"][name][fired], Yd[fired], rtol=0, atol=1e-12)
            assert np.allclose(r["Y"][name][~fired], Ys[~fired], rtol=0, atol=1e-12)


def pin_paper_speedups(O, rows):
    # Eq. (speedup) against every (fast %, S_eff) pair the paper prints; the printed fast-path
    # percentage is itself rounded to 0.1 %, so the printed S must lie in the image of that interval.
    assert len(rows) == 27
    for model, d, k, eps, fpct, sprinted in rows:
        d, k, f, s = int(d), int(k), float(fpct) / 100.0, float(sprinted)
        lo = O.effective_speedup(max(f - 0.0005, 0.0), d, k)
        hi = O.effective_speedup(min(f + 0.0005, 1.0), d, k)
        assert lo - 0.05 - 1e-9 <= s <= hi + 0.05 + 1e-9, (model, k, eps, lo, hi, s)
    assert abs(O.effective_speedup(1.0, 4096, 256) - 16.0) < 1e-12
    assert abs(O.effective_speedup(0.0, 4096, 256) - 1.0) < 1e-12
    # model-wide value = harmonic mean weighted by weight volume = total dense volume / total gated volume
    layers = [(0.9, 4096, 256, 3.0), (0.5, 4096, 128, 1.0)]
    by_hand = 4.0 / (3.0 * (0.9 / 16 + 0.1) + 1.0 * (0.5 / 32 + 0.5))
    assert abs(O.model_speedup(layers) - by_hand) < 1e-12


def pin_paper_closed_forms(O, rows):
    vals = {name: (float(v), float(tol)) for name, v, tol in rows}
    v, tol = vals["basis_storage_bytes_gptj"]
    assert abs(2 * O.basis_storage_elems(28, 4096, 256) - v) <= tol
    v, tol = vals["image_storage_bytes_gptj_printed"]
    assert abs(2 * O.image_storage_elems([4096, 4096, 4096, 4096, 16384], 28, 256) - v) <= tol
    v, tol = vals["effective_params_gptj"]
    # one "layer" holding all 6e9 parameters: N_W d_out d = 6e9 with d = 4096
    assert abs(O.effective_params([(1, 6e9 / 4096, 4096, 256, 0.998)]) - v) <= tol
    v, tol = vals["max_speedup_gptj_k256"]
    assert abs(O.effective_speedup(1.0, 4096, 256) - v) <= tol
    # f = 1 => P_eff is d/k smaller than the full count
    assert abs(O.effective_params([(6, 4096, 4096, 256, 1.0)]) * 16 - 6 * 4096 * 4096) < 1e-6


def pin_alg1_mixed_mask(O):
    # Algorithm 1 as printed, both branches in one call: a fired token gets W x, an un-fired one M c of
    # *its own* coefficients.  Expected values are exactly rounded loop sums that never call the oracle.
    rng = np.random.default_rng(31)
    d, k, m, B = 11, 3, 4, 5
    U, _ = np.linalg.qr(rng.standard_normal((d, k)))
    X = rng.standard_normal((B, d)) * np.array([1.0, 3.0, 0.5, 2.0, 7.0])[:, None]   # tokens differ in size
    W = rng.standard_normal((m, d))
    mask = np.array([0, 1, 0, 0, 1], dtype=np.uint8)
    WU = _fsum_matmul(W, U)
    C = np.array([_fsum_matvec(U.T, X[t]) for t in range(B)])
    Y = O.gated_linear_alg1(W, WU, C, X, mask)
    assert Y.shape == (B, m)
    for t in range(B):
        yexp = _fsum_matvec(W, X[t]) if mask[t] else _fsum_matvec(WU, C[t])
        assert np.allclose(Y[t], yexp, rtol=0, atol=1e-13), t
    # the un-fired rows differ from token to token and from the dense product (the fast path approximates)
    assert np.linalg.norm(Y[0] - Y[2]) > 1e-3 and np.linalg.norm(Y[0] - _fsum_matvec(W, X[0])) > 1e-3
    # hand-worked (same numbers as pin_hand_worked_2d): un-fired gives M c = (4.84, 11, 17.16)
    U2, X2 = np.array([[0.6], [0.8]]), np.array([[1.0, 2.0], [1.0, 2.0]])
    W2 = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    Y2 = O.gated_linear_alg1(W2, np.array([[2.2], [5.0], [7.8]]), np.array([[2.2], [2.2]]), X2, np.array([0, 1], dtype=np.uint8))
    assert np.allclose(Y2, [[4.84, 11.0, 17.16], [5.0, 11.0, 17.0]], rtol=0, atol=1e-13)


def pin_residual_ratio_zero_input(O):
    # x = 0 gives 0/0; the reading taken is rho := 0 (and the gate does not fire).  Other entries are plain quotients.
    rho = O.residual_ratio(np.array([0.0, 0.3, 0.0, 2.0]), np.array([0.0, 0.6, 5.0, 2.0]))
    assert rho.tolist() == [0.0, 0.5, 0.0, 1.0]
    assert O.residual_ratio(np.zeros(3), np.zeros(3)).tolist() == [0.0, 0.0, 0.0]


def pin_single_pass_residual_norm(O):
    # Hand-worked with a basis that is NOT unit length: U = 1.1 (3/5, 4/5)^T, x = (1, 2).
    # c = 2.42, U c = (1.5972, 2.1296), r = (-0.5972, -0.1296), |r|^2 = 0.373444.
    # E = U^T U - 1 = 0.21; |x|^2 - c^2 + c E c = 5 - 5.8564 + 1.229844 = 0.373444.
    U = np.array([[0.66], [0.88]])
    E = O.gram_defect(U)
    assert E.shape == (1, 1) and abs(E[0, 0] - 0.21) < 1e-15
    x = np.array([1.0, 2.0])
    assert abs(O.residual_norm_single_pass(x, np.array([2.42]), E) - math.sqrt(0.373444)) < 1e-14
    # The defect of an axis-aligned, scaled basis is diagonal with entries s_j^2 - 1 and zero elsewhere.
    S = np.zeros((5, 3))
    S[[4, 0, 2], [0, 1, 2]] = [2.0, 0.5, 1.0]
    assert np.array_equal(O.gram_defect(S), np.diag([3.0, -0.75, 0.0]))
    # Any stored basis (a bf16-rounded orthonormal one, and a plain random matrix far from orthonormal):
    # the one-pass value equals the norm of the residual formed explicitly with exactly rounded loop sums.
    rng = np.random.default_rng(77)
    d, k = 13, 4
    Q, _ = np.linalg.qr(rng.standard_normal((d, k)))
    for U in (O.widen(wl.store(Q, "bf16"), "bf16"), 0.4 * rng.standard_normal((d, k))):
        E = O.gram_defect(U)
        assert np.allclose(E, _fsum_matmul(U.T, U) - np.eye(k), rtol=0, atol=1e-15)
        assert np.allclose(E, E.T, rtol=0, atol=0)
        X = rng.standard_normal((3, d))
        C, rn, xn = O.project_single_pass(U, E, X)
        for t in range(3):
            c = _fsum_matvec(U.T, X[t])
            r = X[t] - _fsum_matvec(U, c)
            assert np.allclose(C[t], c, rtol=0, atol=1e-14)
            assert abs(rn[t] - math.sqrt(math.fsum(v * v for v in r))) < 1e-13
            assert abs(xn[t] - math.sqrt(math.fsum(v * v for v in X[t]))) < 1e-14
    # x in the span of an orthonormal basis: the value under the root is round-off of either sign; clamped, never NaN
    x = Q @ rng.standard_normal(k)
    v = O.residual_norm_single_pass(x, Q.T @ x, O.gram_defect(Q))
    assert 0.0 <= v < 1e-7
    # a value under the root that rounding made negative gives 0, not NaN: |x|^2 = 25, c^2 = 25 + 1e-8
    assert O.residual_norm_single_pass(np.array([3.0, 4.0]), np.array([5.000000001]), np.zeros((1, 1))) == 0.0


def pin_round_to_storage(O):
    # bf16 has 8 significand bits: 1 + 2^-8 is a tie between 1 and 1 + 2^-7 and goes to the even code (1.0);
    # 1 + 3 * 2^-8 is a tie between 1 + 2^-7 (odd) and 1 + 2^-6 (even) and goes up.
    vals = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -40, 1.0 + 3 * 2.0 ** -8, -(1.0 + 3 * 2.0 ** -8),
                     0.0, 2.0 ** -8 * (1 - 2.0 ** -9), 1.0 - 2.0 ** -30])
    codes = O.round_to_storage(vals, "bf16")
    assert codes.dtype == np.uint16
    assert codes.tolist() == [0x3F80, 0x3F80, 0x3F81, 0x3F82, 0xBF82, 0x0000, 0x3B80, 0x3F80]
    # a double-rounding trap: just above a bf16 tie by less than half an fp32 ulp must still round up
    assert O.round_to_storage(np.array([1.0 + 2.0 ** -8 + 2.0 ** -30]), "bf16").tolist() == [0x3F81]
    # every bf16 value is a fixed point
    allc = np.arange(0x0080, 0x7F80, 37, dtype=np.uint16)
    assert np.array_equal(O.round_to_storage(O.widen(allc, "bf16"), "bf16"), allc)
    f = O.round_to_storage(np.array([0.1, -2.5]), "f32")
    assert f.dtype == np.float32 and f.tolist() == [np.float32(0.1), np.float32(-2.5)]


def pin_dgks_extension(O):
    # Hand-worked: U = e1 in R^3, x = (1, 1, 0): r = (0, 1, 0), the new direction is e2, both norms are 1.
    U = np.array([[1.0], [0.0], [0.0]])
    u, n1, n2 = O.dgks_direction(U, np.array([1.0, 1.0, 0.0]))
    assert u.tolist() == [0.0, 1.0, 0.0] and n1 == 1.0 and n2 == 1.0
    # x already in the span: zero direction, zero norms
    u, n1, n2 = O.dgks_direction(U, np.array([-3.0, 0.0, 0.0]))
    assert u.tolist() == [0.0, 0.0, 0.0] and n1 == 0.0 and n2 == 0.0
    # Against a library routine: the new direction is, up to the sign convention, the last column of the QR
    # factorisation of [U, x]; the extended basis stays orthonormal and x lies in its span.
    rng = np.random.default_rng(5)
    d, k = 17, 5
    Q, _ = np.linalg.qr(rng.standard_normal((d, k)))
    x = rng.standard_normal(d)
    u, n1, n2 = O.dgks_direction(Q, x)
    Q2, R2 = np.linalg.qr(np.column_stack([Q, x]))
    q = Q2[:, k] * np.sign(R2[k, k])
    assert np.allclose(u, q, rtol=0, atol=1e-13)
    assert abs(n1 - abs(R2[k, k])) < 1e-13 and abs(n2 - n1) < 1e-13
    V = np.column_stack([Q, u])
    assert np.abs(_fsum_matmul(V.T, V) - np.eye(k + 1)).max() < 1e-14
    assert np.linalg.norm(x - V @ (V.T @ x)) < 1e-13 * np.linalg.norm(x)
    # "Twice is enough": x nearly in the span (residual 1e-9 of |x|), one pass alone leaves a direction that is
    # not orthogonal to U at working precision; with the second pass it is.
    n = rng.standard_normal(d)
    n -= Q @ (Q.T @ n)
    n /= np.linalg.norm(n)
    x = Q @ rng.standard_normal(k) * 1e3 + 1e-6 * n
    u, n1, n2 = O.dgks_direction(Q, x)
    assert np.abs(Q.T @ u).max() < 1e-14 and abs(np.linalg.norm(u) - 1.0) < 1e-14
    assert abs(u @ n) > 1 - 1e-6
    # Proposition "Monotonicity" on the extended basis: the residual ratio of any token does not grow.
    Y = rng.standard_normal((6, d))
    for y in Y:
        before = np.linalg.norm(y - Q @ (Q.T @ y))
        after = np.linalg.norm(y - V @ (V.T @ y))
        assert after <= before + 1e-14


def pin_extend_basis_array(O):
    rng = np.random.default_rng(8)
    d, K, k, m = 24, 6, 3, 7
    Q, _ = np.linalg.qr(rng.standard_normal((d, k)))
    for dt in ("f32", "bf16"):
        store = np.zeros((d, K), dtype=np.float32 if dt == "f32" else np.uint16)
        store[:, :k] = Q.astype(np.float32) if dt == "f32" else wl.store(Q, "bf16")
        U = O.widen(store, dt)
        x = rng.standard_normal(d)
        rho = np.linalg.norm(x - U @ (U.T @ x)) / np.linalg.norm(x)   # well away from 0 and 1
        # below the threshold, at zero input, and at full capacity nothing changes
        for args in ((store, dt, k, x, rho * 1.01), (store, dt, k, np.zeros(d), 0.0)):
            out, k2, ext = O.extend_basis(*args)
            assert not ext and k2 == k and out is store
        full = store.copy()
        full[:, k:] = store[:, :1]
        out, k2, ext = O.extend_basis(full, dt, K, x, 0.0)
        assert not ext and k2 == K
        # at the threshold (>=, like the gate) the basis grows by one stored column; the others are untouched
        out, k2, ext = O.extend_basis(store, dt, k, x, np.float32(rho * (1 - 1e-6)))
        assert ext and k2 == k + 1
        assert np.array_equal(out[:, :k], store[:, :k]) and not out[:, k + 1:].any()
        unew = O.widen(out, dt)[:, k]
        # it is the rounded normalised residual: within half a unit in the last place of the exact direction
        r = x - U @ (U.T @ x)
        r = r - U @ (U.T @ r)
        exact = r / np.linalg.norm(r)
        ulp = 2.0 ** -24 if dt == "f32" else 2.0 ** -8
        assert np.all(np.abs(unew - exact) <= ulp * np.abs(exact) + 1e-300)
        # x now has (up to storage rounding) no residual, and no token's ratio grew
        V = O.widen(out, dt)
        assert np.linalg.norm(x - V @ (V.T @ x)) <= 4 * ulp * np.linalg.norm(x) + (0.05 if dt == "bf16" else 1e-6) * rho * np.linalg.norm(x)
        # the image append: column k of M becomes W u_new for the STORED column, the rest is untouched, so M = W U
        W = rng.standard_normal((m, d))
        M = np.zeros((m, K))
        M[:, :k] = _fsum_matmul(W, U[:, :k])
        M2 = O.extend_image(M, k, W, unew)
        assert np.array_equal(M2[:, :k], M[:, :k]) and not M2[:, k + 1:].any()
        assert np.allclose(M2, _fsum_matmul(W, V), rtol=0, atol=1e-13)


def pin_extend_threshold(O):
    # The threshold compares like the gate: >= , against tau rounded to fp32.
    U1 = np.zeros((2, 2), dtype=np.float32)
    U1[0, 0] = 1.0
    # x orthogonal to the basis: ratio exactly 1, tau = 1 extends (a strict comparison would not)
    _, k, ext = O.extend_basis(U1, "f32", 1, np.array([0.0, 2.0]), 1.0)
    assert ext and k == 2
    # x = (4, 3): r = (0, 3), ratio = 3/5, the double nearest to 0.6; fp32(0.6) = 0.60000002... is larger: no growth
    _, k, ext = O.extend_basis(U1, "f32", 1, np.array([4.0, 3.0]), 0.6)
    assert not ext and k == 1
    # ratio 0.699999995 lies between fp32(0.7) = 0.69999998807... and 0.7: grows only because tau is rounded to fp32
    rr = 0.699999995
    _, k, ext = O.extend_basis(U1, "f32", 1, np.array([math.sqrt(1.0 - rr * rr), rr]), 0.7)
    assert ext and k == 2


def pin_track_basis(O):
    # Tokens drawn from a 3-dimensional subspace plus one outlier direction: started empty with capacity 8 the
    # tracker grows to exactly rank 4 (three from the subspace, one for the outlier) and then stops growing.
    rng = np.random.default_rng(21)
    d, K = 16, 8
    B3, _ = np.linalg.qr(rng.standard_normal((d, 4)))
    coef = rng.standard_normal((12, 3))
    X = coef @ B3[:, :3].T
    X[7] += 2.0 * B3[:, 3]
    store = np.zeros((d, K), dtype=np.float32)
    out, k, grew = O.track_basis(store, "f32", 0, X, 1e-3)
    assert k == 4 and grew == [0, 1, 2, 7]
    V = O.widen(out, "f32")[:, :k]
    assert np.abs(V.T @ V - np.eye(k)).max() < 1e-6 and not out[:, k:].any()
    for x in X:
        assert np.linalg.norm(x - V @ (V.T @ x)) < 1e-5 * np.linalg.norm(x)
    # capacity 2: growth stops at 2 and later tokens keep their residual
    out2, k2, grew2 = O.track_basis(np.zeros((d, 2), dtype=np.float32), "f32", 0, X, 1e-3)
    assert k2 == 2 and grew2 == [0, 1]
    # the cascade (Section 5.3): started from a basis that already spans the subspace only the outlier extends it
    warm = np.zeros((d, K), dtype=np.float32)
    warm[:, :3] = B3[:, :3].astype(np.float32)
    out3, k3, grew3 = O.track_basis(warm, "f32", 3, X, 1e-3)
    assert k3 == 4 and grew3 == [7]


PINS = [
    pin_single_pass_residual_norm,
    pin_round_to_storage,
    pin_dgks_extension,
    pin_extend_basis_array,
    pin_extend_threshold,
    pin_track_basis,
    pin_hand_worked_2d,
    pin_axis_aligned_basis,
    pin_brute_force_tiny,
    pin_orthogonality_and_pythagoras,
    pin_designed_rho,
    pin_full_rank_basis,
    pin_monotone_in_k,
    pin_all_fire_is_dense,
    pin_none_fire_is_static_projection,
    pin_error_bound,
    pin_gate_boundary,
    pin_batch_equals_per_token,
    pin_widen,
    pin_stack,
    pin_alg1_mixed_mask,
    pin_residual_ratio_zero_input,
]


# ---- the FP8 image (Section 7 "Combination with quantization"; format reading: OCP E4M3, power-of-two row scales) ----
def _fp8_grid():
    """All finite E4M3 magnitudes from the definition, ascending, with their codes -- built without the oracle."""
    vals = []
    for e in range(16):
        for m in range(8):
            if e == 15 and m == 7:
                continue
            v = (m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
            vals.append((v, (e << 3) | m))
    return vals


def pin_fp8_code_values(O, rows):
    codes = np.array([int(r[0], 16) for r in rows], dtype=np.uint8)
    want = np.array([float(r[1]) for r in rows])
    got = O.fp8_e4m3_decode(codes)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]) | (codes[ok] >= 0x80))


def pin_fp8_decode_all_codes(O):
    grid = _fp8_grid()
    got = O.fp8_e4m3_decode(np.arange(256, dtype=np.uint8))
    for v, c in grid:
        assert got[c] == v and got[c | 0x80] == -v
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF])
    assert len(grid) == 127 and max(v for v, _ in grid) == 448.0


def pin_fp8_encode_is_nearest_ties_even(O):
    grid = _fp8_grid()
    vals = np.array([v for v, _ in grid])
    codes = np.array([c for _, c in grid])
    # every code value encodes to itself, with the sign bit
    assert np.array_equal(O.fp8_e4m3_encode(vals), codes.astype(np.uint8))
    assert np.array_equal(O.fp8_e4m3_encode(-vals[1:]), (codes[1:] | 0x80).astype(np.uint8))
    # exact midpoints go to the neighbour with the even code; a hair to either side goes to that side
    mid = 0.5 * (vals[:-1] + vals[1:])
    got = O.fp8_e4m3_encode(mid)
    even = np.where(codes[:-1] % 2 == 0, codes[:-1], codes[1:])
    assert np.array_equal(got, even.astype(np.uint8))
    assert np.array_equal(O.fp8_e4m3_encode(np.nextafter(mid, 0.0)), codes[:-1].astype(np.uint8))
    assert np.array_equal(O.fp8_e4m3_encode(np.nextafter(mid, np.inf)), codes[1:].astype(np.uint8))
    # brute force over random magnitudes spanning subnormal to maximum: the chosen code is a nearest one
    rng = np.random.default_rng(5)
    x = np.exp(rng.uniform(np.log(2.0 ** -12), np.log(448.0), 4000)) * rng.choice([-1.0, 1.0], 4000)
    got = O.fp8_e4m3_encode(x)
    dist = np.abs(np.abs(x)[:, None] - vals[None, :])
    best = dist.min(axis=1)
    chosen = np.abs(O.fp8_e4m3_decode(got))
    assert np.array_equal(np.abs(np.abs(x) - chosen), best)
    assert np.array_equal(got >= 0x80, x < 0)
    # monotone
    xs = np.sort(np.abs(x))
    assert np.all(np.diff(O.fp8_e4m3_encode(xs).astype(int)) >= 0)


def pin_fp8_saturation_and_nan(O):
    got = O.fp8_e4m3_encode(np.array([449.0, 464.0, 1e6, -1e6, np.inf, -np.inf, np.nan, 0.0, -0.0, 2.0 ** -10, 2.0 ** -10 * 1.01]))
    assert list(got) == [0x7E, 0x7E, 0x7E, 0xFE, 0x7E, 0xFE, 0x7F, 0x00, 0x80, 0x00, 0x01]


def pin_fp8_matches_library_cast(O):
    # PyTorch's CPU cast to float8_e4m3fn is an independent implementation of the same encoding
    # (round to nearest even); compared inside the finite range, where saturation does not matter
    import torch
    rng = np.random.default_rng(6)
    x = (rng.standard_normal(50000) * np.exp(rng.uniform(-12, 6, 50000))).clip(-448, 448).astype(np.float32)
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(O.fp8_e4m3_encode(x), want)
    back = torch.from_numpy(want).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(O.fp8_e4m3_decode(want), back)


def pin_fp8_row_scale(O):
    M = np.array([[448.0, 1.0], [448.0000001, 0.0], [224.0, -3.0], [-224.0000001, 3.0], [0.0, 0.0], [1e-30, 0.0], [-7.0, 6.0]])
    s = O.fp8_row_scale(M)
    assert list(s) == [1.0, 2.0, 0.5, 1.0, 1.0, 2.0 ** -108, 2.0 ** -6]
    assert list(O.fp8_row_scale(np.array([[np.inf, 3.5], [np.nan, -896.0], [np.nan, np.inf]]))) == [2.0 ** -7, 2.0, 1.0]
    rng = np.random.default_rng(7)
    M = rng.standard_normal((64, 32)) * np.exp(rng.uniform(-20, 20, (64, 1)))
    s = O.fp8_row_scale(M)
    top = np.abs(M).max(axis=1) / s
    assert np.all((top > 224.0) & (top <= 448.0))
    assert np.all(np.log2(s) == np.round(np.log2(s)))


def pin_fp8_quantization_error(O):
    # relative error at most half a code step (2^-4) on elements in the normal range of their row,
    # absolute error at most half the subnormal step below it; the image product inherits the bound
    rng = np.random.default_rng(8)
    m, k = 48, 40
    M = rng.standard_normal((m, k)) * np.exp(rng.uniform(-3, 3, (m, k)))
    codes, s = O.quantize_image_fp8(M)
    Mh = O.dequantize_image_fp8(codes, s)
    normal = np.abs(M) >= s[:, None] * 2.0 ** -6
    assert np.all(np.abs(Mh - M)[normal] <= 2.0 ** -4 * np.abs(M)[normal])
    assert np.all(np.abs(Mh - M)[~normal] <= s[:, None].repeat(k, 1)[~normal] * 2.0 ** -10)
    assert np.any(np.abs(Mh - M)[normal] > 2.0 ** -6 * np.abs(M)[normal])   # it is 3 bits, not more
    c = rng.standard_normal(k)
    bound = 2.0 ** -4 * (np.abs(M) @ np.abs(c)) + s * 2.0 ** -10 * np.sum(np.abs(c))
    assert np.all(np.abs(Mh @ c - M @ c) <= bound)
    # a matrix of code values is reproduced exactly, whatever the row scale
    vals = np.array([v for v, _ in _fp8_grid()])[1:]
    E = rng.choice(vals, (8, 16)) * rng.choice([-1.0, 1.0], (8, 16)) * (2.0 ** rng.integers(-9, 9, (8, 1)))
    E[:, 0] = 448.0 * (2.0 ** np.round(np.log2(np.abs(E).max(axis=1) / 448.0) + 0.49999))  # pin the row maximum to a code value
    codes, s = O.quantize_image_fp8(E)
    assert np.array_equal(O.dequantize_image_fp8(codes, s), E)


FP8_PINS = [
    pin_fp8_decode_all_codes,
    pin_fp8_encode_is_nearest_ties_even,
    pin_fp8_saturation_and_nan,
    pin_fp8_matches_library_cast,
    pin_fp8_row_scale,
    pin_fp8_quantization_error,
]
