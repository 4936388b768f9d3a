"""Plant plausible mistakes in copies of the CPU oracle and require that the pins catch each one.

Every mutant is the oracle's own source with one line changed (a dropped term, a wrong sign, a
transposed operand, a wrong index, an off-by-one comparison).  All of this runs on the CPU.
"""
import os
import types

import pytest

from conftest import ROOT, read_golden
from oracle_pins import FP8_PINS, PINS, pin_fp8_code_values, pin_paper_closed_forms, pin_paper_speedups

SRC = open(os.path.join(ROOT, "oracle", "gsi_oracle.py")).read()

MUTANTS = [
    ("c_uses_U_not_UT", "c = U.T @ x ", "c = (x @ U[:, ::-1]) "),
    ("residual_sign", "r = x - U @ c ", "r = x + U @ c "),
    ("residual_dropped", "r = x - U @ c ", "r = x.copy() "),
    ("rnorm_no_sqrt", "rnorm[t] = np.sqrt(np.sum(r * r))", "rnorm[t] = np.sum(r * r)"),
    ("rnorm_l1", "rnorm[t] = np.sqrt(np.sum(r * r))", "rnorm[t] = np.sum(np.abs(r))"),
    ("xnorm_of_r", "xnorm[t] = np.sqrt(np.sum(x * x))", "xnorm[t] = np.sqrt(np.sum(r * r))"),
    ("rho_inverted", "rho[nz] = rnorm[nz] / xnorm[nz]", "rho[nz] = xnorm[nz] / rnorm[nz].clip(1e-300)"),
    ("gate_strict", "& (rho >= eps64)", "& (rho > eps64)"),
    ("gate_reversed", "& (rho >= eps64)", "& (rho < eps64)"),
    ("gate_eps_fp64", "eps64 = float(np.float32(eps))", "eps64 = float(eps)"),
    ("gate_zero_x_fires", "fired = (np.asarray(xnorm) > 0) & (rho >= eps64)", "fired = (rho >= eps64)"),
    ("idx_descending", "idx = np.nonzero(fired)[0].astype(np.int32)", "idx = np.nonzero(fired)[0][::-1].astype(np.int32)"),
    ("image_transposed_U", "@ np.asarray(U, dtype=np.float64)\n", "@ np.asarray(U, dtype=np.float64)[:, ::-1]\n"),
    ("image_is_W_slice", "return np.asarray(W, dtype=np.float64) @ np.asarray(U, dtype=np.float64)",
     "return np.asarray(W, dtype=np.float64)[:, : U.shape[1]].copy()"),
    ("fast_term_dropped", "y = M @ C[t] ", "y = 0.0 * (M @ C[t]) "),
    ("slow_term_sign", "y = y + W @ R[t] ", "y = y - W @ R[t] "),
    ("slow_term_always", "if mask[t]:\n            y = y + W @ R[t]", "if True:\n            y = y + W @ R[t]"),
    ("slow_term_never", "if mask[t]:\n            y = y + W @ R[t]", "if False:\n            y = y + W @ R[t]"),
    ("slow_term_uses_wrong_token", "y = y + W @ R[t] ", "y = y + W @ R[0] "),
    ("alg1_branches_swapped", "Y[t] = W @ X[t] if mask[t] else M @ C[t]", "Y[t] = M @ C[t] if mask[t] else W @ X[t]"),
    ("alg1_unfired_uses_first_token", "Y[t] = W @ X[t] if mask[t] else M @ C[t]", "Y[t] = W @ X[t] if mask[t] else M @ C[0]"),
    ("alg1_unfired_doubled", "Y[t] = W @ X[t] if mask[t] else M @ C[t]", "Y[t] = W @ X[t] if mask[t] else 2.0 * (M @ C[t])"),
    ("alg1_fired_uses_image", "Y[t] = W @ X[t] if mask[t] else M @ C[t]", "Y[t] = M @ C[t]"),
    ("rho_one_at_zero_input", "rho = np.zeros_like(rnorm)", "rho = np.ones_like(rnorm)"),
    ("dense_transposed", "Y[t] = W @ X[t]\n    return Y\n\n\ndef gated_linear(", "Y[t] = (W[::-1] @ X[t])\n    return Y\n\n\ndef gated_linear("),
    ("bf16_shift", "<< np.uint32(16)", "<< np.uint32(15)"),
    ("speedup_formula", "return 1.0 / (f / (d / k) + (1.0 - f))", "return 1.0 / (f * (d / k) + (1.0 - f))"),
    ("speedup_kd_swapped", "return 1.0 / (f / (d / k) + (1.0 - f))", "return 1.0 / (f / (k / d) + (1.0 - f))"),
    ("model_speedup_arithmetic_mean", "return vol / sum(v / effective_speedup(f, d, k) for f, d, k, v in layers)",
     "return sum(v * effective_speedup(f, d, k) for f, d, k, v in layers) / vol"),
    ("peff_swapped", "(f * k + (1.0 - f) * d)", "(f * d + (1.0 - f) * k)"),
    ("stack_gate_per_map_wrong_eps", "mask, idx, n = gate(rn, xn, eps)", "mask, idx, n = gate(rn, xn, 2.0 * eps)"),
    ("stack_dense_uses_image", "name: dense_linear(W64, X) for name, W64, _ in g[\"maps\"]", "name: dense_linear(W64, X) * 1.0000001 for name, W64, _ in g[\"maps\"]"),
    ("error_bound_smallest_sv", "compute_uv=False)[0]", "compute_uv=False)[-1]"),
    # the one-pass residual norm
    ("gram_defect_keeps_identity", "return U.T @ U - np.eye(U.shape[1])", "return U.T @ U"),
    ("gram_defect_is_UUT", "return U.T @ U - np.eye(U.shape[1])", "return (U @ U.T)[: U.shape[1], : U.shape[1]] - np.eye(U.shape[1])"),
    ("single_pass_drops_defect_term", "- np.sum(c * c) + c @ (np.asarray(E, dtype=np.float64) @ c)", "- np.sum(c * c)"),
    ("single_pass_defect_sign", "- np.sum(c * c) + c @ (np.asarray(E, dtype=np.float64) @ c)", "- np.sum(c * c) - c @ (np.asarray(E, dtype=np.float64) @ c)"),
    ("single_pass_counts_c_twice", "q = np.sum(x * x) - np.sum(c * c)", "q = np.sum(x * x) - 2.0 * np.sum(c * c)"),
    ("single_pass_no_root", "return float(np.sqrt(max(q, 0.0)))", "return float(max(q, 0.0))"),
    ("single_pass_no_clamp", "return float(np.sqrt(max(q, 0.0)))", "return float(np.sqrt(q))"),
    ("single_pass_xnorm_of_c", "xnorm[t] = np.sqrt(np.sum(X[t] * X[t]))", "xnorm[t] = np.sqrt(np.sum(C[t] * C[t]))"),
    # rounding to storage, rank-1 extension, tracker
    ("round_truncates", "up = (dhi < dlo) | (", "up = (dhi < 0 * dlo) & ("),
    ("round_ties_away", "& (((lo >> np.uint32(16)) & np.uint32(1)) == 1))", "& (((lo >> np.uint32(16)) & np.uint32(1)) >= 0))"),
    ("round_via_fp32_first", "dlo, dhi = np.abs(a - vlo), np.abs(vhi - a)", "dlo, dhi = np.abs(f - vlo), np.abs(vhi - f)"),
    ("dgks_single_pass_only", "r2 = r - U @ s\n", "r2 = r\n"),
    ("dgks_second_pass_sign", "r2 = r - U @ s\n", "r2 = r + U @ s\n"),
    ("dgks_not_normalised", "u = r2 / n2 if n2 > 0", "u = r2 if n2 > 0"),
    ("dgks_normalised_by_first_norm", "u = r2 / n2 if n2 > 0", "u = r2 / max(n1, 1.0) if n2 > 0"),
    ("dgks_direction_is_x", "u = r2 / n2 if n2 > 0", "u = x / np.sqrt(np.sum(x * x)) if n2 > 0"),
    ("extend_strict_threshold", "n1 / xn >= float(np.float32(tau))", "n1 / xn > float(np.float32(tau))"),
    ("extend_threshold_fp64", "n1 / xn >= float(np.float32(tau))", "n1 / xn >= float(tau)"),
    ("extend_ignores_capacity", "and k < K and n2 > 0", "and k <= K and n2 > 0"),
    ("extend_wrong_column", "out[:, k] = round_to_storage(u, udtype)", "out[:, max(k - 1, 0)] = round_to_storage(u, udtype)"),
    ("extend_rank_not_advanced", "return out, k + 1, True", "return out, k, True"),
    ("extend_image_wrong_column", "out[:, k] = np.asarray(W, dtype=np.float64) @", "out[:, k - 1] = np.asarray(W, dtype=np.float64) @"),
    ("extend_image_transposed", "out[:, k] = np.asarray(W, dtype=np.float64) @ np.asarray(u_stored, dtype=np.float64)",
     "out[:, k] = np.asarray(W, dtype=np.float64)[:, ::-1] @ np.asarray(u_stored, dtype=np.float64)"),
    ("track_tests_first_token_only", "U_store, k, ext = extend_basis(U_store, udtype, k, X[t], tau)", "U_store, k, ext = extend_basis(U_store, udtype, k, X[0], tau)"),
    ("track_forgets_growth", "U_store, k, ext = extend_basis(U_store, udtype, k, X[t], tau)", "_, k, ext = extend_basis(U_store, udtype, k, X[t], tau)"),
    # the FP8 image
    ("fp8_bias", "np.exp2((e - 7).astype(np.float64))", "np.exp2((e - 8).astype(np.float64))"),
    ("fp8_subnormal_exponent", "(m / 8.0) * 2.0 ** -6", "(m / 8.0) * 2.0 ** -7"),
    ("fp8_nan_code_is_480", "val = np.where((e == 15) & ((c & 0x7) == 7), np.nan, val)", "val = val + 0.0"),
    ("fp8_sign_dropped", "return sign * val", "return val"),
    ("fp8_round_half_up", "q = np.rint(a / step).astype(np.int64)", "q = np.floor(a / step + 0.5).astype(np.int64)"),
    ("fp8_truncates", "q = np.rint(a / step).astype(np.int64)", "q = np.floor(a / step).astype(np.int64)"),
    ("fp8_no_saturation", "np.minimum(a, FP8_MAX)", "np.minimum(a, 1e30)"),
    ("fp8_subnormal_floor_exponent", "e = np.maximum(e, -6)", "e = np.maximum(e, -7)"),
    ("fp8_carry_lost", "q = np.where(carry, 8, q)", "q = np.where(carry, 15, q)"),
    ("fp8_encode_sign_dropped", "code = np.where(np.signbit(x) & ~nan, code | 0x80, code)", "code = code + 0"),
    ("fp8_scale_uses_largest_normal_480", "FP8_MAX = 448.0", "FP8_MAX = 480.0"),
    ("fp8_scale_not_power_of_two", "scale[i] = 2.0 ** min(max(e, -126), 127)", "scale[i] = a / FP8_MAX"),
    ("fp8_scale_one_binade_large", "scale[i] = 2.0 ** min(max(e, -126), 127)", "scale[i] = 2.0 ** min(max(e + 1, -126), 127)"),
    ("fp8_quantize_ignores_scale", "return fp8_e4m3_encode(M / scale[:, None]), scale", "return fp8_e4m3_encode(M), scale"),
    ("fp8_dequantize_ignores_scale", "return fp8_e4m3_decode(codes) * np.asarray(scale, dtype=np.float64)[:, None]",
     "return fp8_e4m3_decode(codes)"),
]


def _load(src):
    mod = types.ModuleType("oracle_mutant")
    exec(compile(src, "oracle_mutant", "exec"), mod.__dict__)
    return mod


def _caught(O):
    pins = list(PINS) + list(FP8_PINS) + [
        lambda o: pin_fp8_code_values(o, read_golden("fp8_e4m3_values.txt")),
        lambda o: pin_paper_speedups(o, read_golden("paper_speedup_tables.txt")),
        lambda o: pin_paper_closed_forms(o, read_golden("paper_closed_forms.txt")),
    ]
    for pin in pins:
        try:
            pin(O)
        except AssertionError:
            return True
        except Exception:  # a mutant may also break shapes; that counts as caught
            return True
    return False


def test_unmutated_source_passes():
    assert not _caught(_load(SRC))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, old, new):
    assert SRC.count(old) >= 1, f"mutation site for {name} not found in the oracle source"
    assert _caught(_load(SRC.replace(old, new, 1))), f"no pin notices mutant {name}"
