"""The torch-based input generator (used on the GPU for the large report workloads) keeps the recipe of the
NumPy one: orthonormal nested bases, tokens whose residual ratio against the fp64 basis is the designed one,
exact fired counts.  Run here on the CPU (the generator takes any torch device)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle.gsi_oracle as O  # noqa: E402
from paper_2605_03109_amd import workload_device as wd  # noqa: E402


def test_basis_is_orthonormal_and_nested():
    gen = wd.generator(11, device="cpu")
    U = wd.make_basis64(96, 24, gen).numpy()
    assert np.allclose(U.T @ U, np.eye(24), atol=1e-12)
    assert np.allclose(U[:, :8].T @ U[:, :8], np.eye(8), atol=1e-12)  # a leading block is a basis of lower rank


def test_tokens_have_the_designed_residual_ratio_and_fire_pattern():
    eps, p, T, d, k = 0.05, 1.2, 64, 80, 16
    gen = wd.generator(12, device="cpu")
    U = wd.make_basis64(d, k, gen)
    fired = wd.choose_fired(T, 9, gen)
    assert int(fired.sum()) == 9
    X, rho_star = wd.make_tokens(U, fired, eps, p, gen, chunk=17)  # ragged chunks
    assert X.dtype == torch.float32 and X.shape == (T, d)
    C, R, rn, xn = O.project(U.numpy(), X.numpy().astype(np.float64))
    rho = O.residual_ratio(rn, xn)
    assert np.allclose(rho, rho_star.numpy(), rtol=0, atol=2e-7)  # fp32 storage of x
    mask, idx, n = O.gate(rn, xn, eps)
    assert n == 9 and np.array_equal(mask.astype(bool), fired.numpy())
    lo, hi = rho_star[~fired].numpy(), rho_star[fired].numpy()
    assert lo.max() <= 0.8 * eps + 1e-12 and hi.min() >= 1.2 * eps - 1e-12  # 20 % away from the threshold


def test_weight_scale_and_bernoulli_rate():
    gen = wd.generator(13, device="cpu")
    W = wd.make_weight(64, 256, gen)
    assert W.dtype == torch.bfloat16
    assert abs(float(W.float().std()) * 16.0 - 1.0) < 0.05  # entries N(0, 1/d)
    f = wd.bernoulli_fired(20000, 0.15, gen)
    assert abs(float(f.double().mean()) - 0.15) < 0.01
