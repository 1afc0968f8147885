"""Pins for the oracle's sparse-GP criterion (section 3.2): the value against the dense definition
-log N(y | 0, Khat + lam I) + tr(Kff - Khat) / (2 lam) with Khat = Kuf^T Kuu^-1 Kuf written with
numpy, and every gradient against central differences of that dense definition."""
import numpy as np
import pytest


def dense_phi(Kuu, Kuf, kff, y, lam):
    n = y.shape[0]
    Khat = Kuf.T @ np.linalg.solve(Kuu, Kuf)
    C = Khat + lam * np.eye(n)
    sign, logdet = np.linalg.slogdet(2 * np.pi * C)
    return 0.5 * (y @ np.linalg.solve(C, y) + logdet) + (np.sum(kff) - np.trace(Khat)) / (2 * lam)


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


@pytest.mark.parametrize("U,n", [(1, 1), (2, 5), (4, 9), (7, 20)])
def test_sgp_value_is_the_dense_definition(orc, U, n):
    Kuu, Kuf, kff, y, lam = problem(10 + U, U, n)
    out = orc.sgp_criterion(Kuu, Kuf, kff, y, lam)
    ref = dense_phi(Kuu, Kuf, kff, y, lam)
    assert abs(out["phi"] - ref) <= 1e-10 * max(1.0, abs(ref))


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

    gKuf = fd(lambda a: dense_phi(Kuu, a, kff, y, lam), Kuf)
    gy = fd(lambda a: dense_phi(Kuu, Kuf, kff, a, lam), y)
    gk = fd(lambda a: dense_phi(Kuu, Kuf, a, y, lam), kff)
    glam = (dense_phi(Kuu, Kuf, kff, y, lam + h) - dense_phi(Kuu, Kuf, kff, y, lam - h)) / (2 * h)
    # symmetric perturbations of Kuu: the gradient returned is the symmetric one
    gKuu = np.zeros_like(Kuu)
    for i in range(U):
        for j in range(i + 1):
            E = np.zeros_like(Kuu)
            E[i, j] = E[j, i] = 1.0
            d = (dense_phi(Kuu + h * E, Kuf, kff, y, lam) - dense_phi(Kuu - h * E, Kuf, kff, y, lam)) / (2 * h)
            gKuu[i, j] = gKuu[j, i] = d if i == j else d / 2
    rel = lambda a, b: np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-12)
    assert rel(out["Kuf_bar"], gKuf) < 1e-6
    assert rel(out["y_bar"], gy) < 1e-6
    assert rel(out["Kff_diag_bar"], gk) < 1e-6
    assert abs(out["noise_bar"] - glam) < 1e-5 * max(1.0, abs(glam))
    assert rel(out["Kuu_bar"], gKuu) < 1e-5
    assert np.allclose(out["Kuu_bar"], out["Kuu_bar"].T, rtol=0, atol=1e-12)
