"""Pins for the oracle's sparse-GP criterion (section 3.2).  The oracle evaluates the DEFINITION
(dense Nystrom matrix, -log N(y | 0, Q + lam I) + tr(Kff - Q) / (2 lam)); it is pinned against
  * the section's own efficient evaluation (two Cholesky factors of U x U matrices), written here
    with scipy's routines -- a different decomposition of the same quantity;
  * the exact Gaussian-process marginal likelihood from scipy's multivariate normal when the inducing
    points are the data points (Q = Kuu, the trace term vanishes);
  * central differences of the section's evaluation for every gradient."""
import numpy as np
import pytest
from scipy.linalg import cholesky, solve_triangular
from scipy.stats import multivariate_normal


def section_phi(Kuu, Kuf, kff, y, lam):
    """The criterion as section 3.2 evaluates it."""
    n = y.shape[0]
    Lu = cholesky(Kuu, lower=True)
    B = solve_triangular(Lu, Kuf, lower=True)
    A = B @ B.T / lam + np.eye(Kuu.shape[0])
    La = cholesky(A, lower=True)
    w = solve_triangular(La, B @ y, lower=True)
    return ((np.log(2 * np.pi) + np.log(lam)) * n / 2 + np.sum(np.log(np.diag(La))) + y @ y / (2 * lam)
            - w @ w / (2 * lam * lam) - (np.sum(B * B) - np.sum(kff)) / (2 * lam))


def problem(seed, U, n):
    rng = np.random.default_rng(seed)
    X = rng.uniform(-1, 1, size=(n, 2))
    Z = rng.uniform(-1, 1, size=(U, 2))
    k = lambda a, b: np.exp(-0.5 * ((a[:, None, :] - b[None, :, :]) ** 2).sum(-1) / 0.7 ** 2)
    Kuu = k(Z, Z) + 0.05 * np.eye(U)
    Kuf = k(Z, X)
    kff = np.ones(n) + 0.05
    y = rng.standard_normal(n)
    return Kuu, Kuf, kff, y, 0.3


@pytest.mark.parametrize("U,n", [(1, 1), (2, 5), (4, 9), (7, 20), (40, 130)])
def test_sgp_value_matches_the_sections_evaluation(orc, U, n):
    Kuu, Kuf, kff, y, lam = problem(10 + U, U, n)
    out = orc.sgp_criterion(Kuu, Kuf, kff, y, lam)
    ref = section_phi(Kuu, Kuf, kff, y, lam)
    assert abs(out["phi"] - ref) <= 1e-10 * max(1.0, abs(ref))


@pytest.mark.parametrize("n", [1, 6, 25])
def test_sgp_with_inducing_points_at_the_data_is_the_exact_marginal_likelihood(orc, n):
    rng = np.random.default_rng(77 + n)
    X = rng.uniform(-1, 1, size=(n, 2))
    K = np.exp(-0.5 * ((X[:, None, :] - X[None, :, :]) ** 2).sum(-1) / 0.5 ** 2) + 0.2 * np.eye(n)
    y = rng.standard_normal(n)
    lam = 0.4
    out = orc.sgp_criterion(K, K, np.diag(K).copy(), y, lam)
    ref = -multivariate_normal(mean=np.zeros(n), cov=K + lam * np.eye(n)).logpdf(y)
    assert abs(out["phi"] - ref) <= 1e-10 * max(1.0, abs(ref))
    # and y_bar = (K + lam I)^-1 y, the gradient of that negative log density
    assert np.allclose(out["y_bar"], np.linalg.solve(K + lam * np.eye(n), y), rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("U,n", [(1, 2), (3, 6), (5, 11)])
def test_sgp_gradient_finite_differences(orc, U, n):
    Kuu, Kuf, kff, y, lam = problem(20 + U, U, n)
    out = orc.sgp_criterion(Kuu, Kuf, kff, y, lam)
    h = 1e-6

    def fd(f, x):
        g = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            xp, xm = x.copy(), x.copy()
            xp[idx] += h
            xm[idx] -= h
            g[idx] = (f(xp) - f(xm)) / (2 * h)
        return g

    gKuf = fd(lambda a: section_phi(Kuu, a, kff, y, lam), Kuf)
    gy = fd(lambda a: section_phi(Kuu, Kuf, kff, a, lam), y)
    gk = fd(lambda a: section_phi(Kuu, Kuf, a, y, lam), kff)
    glam = (section_phi(Kuu, Kuf, kff, y, lam + h) - section_phi(Kuu, Kuf, kff, y, lam - h)) / (2 * h)
    # symmetric perturbations of Kuu: the gradient returned is the symmetric one
    gKuu = np.zeros_like(Kuu)
    for i in range(U):
        for j in range(i + 1):
            E = np.zeros_like(Kuu)
            E[i, j] = E[j, i] = 1.0
            d = (section_phi(Kuu + h * E, Kuf, kff, y, lam) - section_phi(Kuu - h * E, Kuf, kff, y, lam)) / (2 * h)
            gKuu[i, j] = gKuu[j, i] = d if i == j else d / 2
    rel = lambda a, b: np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-12)
    assert rel(out["Kuf_bar"], gKuf) < 1e-6
    assert rel(out["y_bar"], gy) < 1e-6
    assert rel(out["Kff_diag_bar"], gk) < 1e-6
    assert abs(out["noise_bar"] - glam) < 1e-5 * max(1.0, abs(glam))
    assert rel(out["Kuu_bar"], gKuu) < 1e-5
    assert np.allclose(out["Kuu_bar"], out["Kuu_bar"].T, rtol=0, atol=1e-12)
