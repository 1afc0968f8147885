"""Pins for the oracle's trmm / trsm / syrk backward rules (section 4.2 and the appendix's
"trsm" and "trmm" derivations): finite differences of a forward pass written here with numpy,
the first-order identity <Bbar, dB> = <Abar, dA> + <Lbar, dL> with dB from the forward-mode
derivative, dense closed forms, structure.  Nothing here calls the oracle to produce a reference.
"""
import itertools

import numpy as np
import pytest

FLAGS = list(itertools.product([True, False], [False, True], [False, True]))  # lower, trans, rightside


def rand_tri(rng, n, lower):
    T = rng.standard_normal((n, n)) * 0.3
    T = np.tril(T) if lower else np.triu(T)
    idx = np.arange(n)
    T[idx, idx] = 1.0 + rng.uniform(0.0, 1.0, size=n)
    return T


def op(T, trans):
    return T.T if trans else T


def fwd_trmm(T, A, trans, rightside, alpha):
    return alpha * (A @ op(T, trans) if rightside else op(T, trans) @ A)


def fwd_trsm(T, A, trans, rightside, alpha):
    Ti = np.linalg.inv(op(T, trans))
    return alpha * (A @ Ti if rightside else Ti @ A)


def fd_gradients(fwd, T, A, Bbar, lower, h=1e-6):
    """Central differences of phi = <Bbar, fwd(T, A)> in every entry of A and of T's triangle."""
    gA = np.zeros_like(A)
    for idx in np.ndindex(*A.shape):
        Ap, Am = A.copy(), A.copy()
        Ap[idx] += h
        Am[idx] -= h
        gA[idx] = (np.sum(Bbar * fwd(T, Ap)) - np.sum(Bbar * fwd(T, Am))) / (2 * h)
    n = T.shape[0]
    gT = np.zeros_like(T)
    for i in range(n):
        for j in range(n):
            if (i >= j) if lower else (i <= j):
                Tp, Tm = T.copy(), T.copy()
                Tp[i, j] += h
                Tm[i, j] -= h
                gT[i, j] = (np.sum(Bbar * fwd(Tp, A)) - np.sum(Bbar * fwd(Tm, A))) / (2 * h)
    return gA, gT


def relerr(x, ref):
    return np.linalg.norm(np.asarray(x) - ref) / max(np.linalg.norm(ref), 1e-300)


@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("n,m", [(1, 1), (4, 3), (7, 5)])
def test_trmm_backward_finite_differences(orc, lower, trans, rightside, n, m):
    rng = np.random.default_rng(300 + 10 * n + m)
    T = rand_tri(rng, n, lower)
    A = rng.standard_normal((m, n) if rightside else (n, m))
    Bbar = rng.standard_normal(A.shape)
    alpha = 1.5
    gA, gT = fd_gradients(lambda t, a: fwd_trmm(t, a, trans, rightside, alpha), T, A, Bbar, lower)
    Abar, Lbar = orc.trmm_backward(T, A, Bbar, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    assert relerr(Abar, gA) < 1e-7
    assert relerr(Lbar, gT) < 1e-7
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    assert np.all(Lbar[other] == 0.0)


@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("n,m", [(1, 1), (4, 3), (7, 5)])
def test_trsm_backward_finite_differences(orc, lower, trans, rightside, n, m):
    rng = np.random.default_rng(400 + 10 * n + m)
    T = rand_tri(rng, n, lower)
    A = rng.standard_normal((m, n) if rightside else (n, m))
    Bbar = rng.standard_normal(A.shape)
    alpha = 0.75
    B = fwd_trsm(T, A, trans, rightside, alpha)
    gA, gT = fd_gradients(lambda t, a: fwd_trsm(t, a, trans, rightside, alpha), T, A, Bbar, lower)
    Abar, Lbar = orc.trsm_backward(T, B, Bbar, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    assert relerr(Abar, gA) < 1e-6
    assert relerr(Lbar, gT) < 1e-6
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    assert np.all(Lbar[other] == 0.0)


@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
def test_trsm_backward_dense_closed_form_and_paper_cases(orc, lower, trans, rightside):
    """The four printed cases (and their upper-factor twins) written out with dense inverses."""
    rng = np.random.default_rng(77)
    n, m = 9, 6
    T = rand_tri(rng, n, lower)
    A = rng.standard_normal((m, n) if rightside else (n, m))
    Bbar = rng.standard_normal(A.shape)
    B = fwd_trsm(T, A, trans, rightside, 1.0)
    Tinv = np.linalg.inv(T)
    if not rightside:
        Ab = (Tinv if trans else Tinv.T) @ Bbar            # L^-T Bbar | L^-1 Bbar
        G = (B @ Ab.T) if trans else (Ab @ B.T)             # B Abar^T | Abar B^T
    else:
        Ab = Bbar @ (Tinv if trans else Tinv.T)             # Bbar L^-T | Bbar L^-1
        G = (Ab.T @ B) if trans else (B.T @ Ab)             # Abar^T B | B^T Abar
    Lb = -(np.tril(G) if lower else np.triu(G))
    Abar, Lbar = orc.trsm_backward(T, B, Bbar, lower=lower, trans=trans, rightside=rightside)
    assert relerr(Abar, Ab) < 1e-12
    assert relerr(Lbar, Lb) < 1e-12


@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
def test_trmm_backward_dense_closed_form_and_paper_cases(orc, lower, trans, rightside):
    rng = np.random.default_rng(78)
    n, m = 8, 5
    T = rand_tri(rng, n, lower)
    A = rng.standard_normal((m, n) if rightside else (n, m))
    Bbar = rng.standard_normal(A.shape)
    if not rightside:
        Ab = (T if trans else T.T) @ Bbar                   # L^T Bbar | L Bbar
        G = (A @ Bbar.T) if trans else (Bbar @ A.T)
    else:
        Ab = Bbar @ (T if trans else T.T)
        G = (Bbar.T @ A) if trans else (A.T @ Bbar)
    Lb = np.tril(G) if lower else np.triu(G)
    Abar, Lbar = orc.trmm_backward(T, A, Bbar, lower=lower, trans=trans, rightside=rightside)
    assert relerr(Abar, Ab) < 1e-13
    assert relerr(Lbar, Lb) < 1e-13


@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
def test_trsm_backward_first_order_identity(orc, lower, trans, rightside):
    """<Bbar, dB> = <Abar, dA> + <Lbar, dL> with dB = t(L)^-1 (alpha dA - t(dL) B) (left) or
    (alpha dA - B t(dL)) t(L)^-1 (right), the differential the appendix starts from."""
    rng = np.random.default_rng(79)
    n, m, alpha = 11, 4, 1.25
    T = rand_tri(rng, n, lower)
    A = rng.standard_normal((m, n) if rightside else (n, m))
    Bbar = rng.standard_normal(A.shape)
    dA = rng.standard_normal(A.shape)
    dT = rng.standard_normal((n, n))
    dT = np.tril(dT) if lower else np.triu(dT)
    B = fwd_trsm(T, A, trans, rightside, alpha)
    Ti = np.linalg.inv(op(T, trans))
    dB = (alpha * dA - B @ op(dT, trans)) @ Ti if rightside else Ti @ (alpha * dA - op(dT, trans) @ B)
    Abar, Lbar = orc.trsm_backward(T, B, Bbar, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    lhs = np.sum(Bbar * dB)
    rhs = np.sum(Abar * dA) + np.sum(Lbar * dT)
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
def test_backward_ops_ignore_the_other_triangle_and_batch(orc, lower, trans, rightside):
    rng = np.random.default_rng(80)
    n, m, batch = 6, 3, 4
    Ts = np.stack([rand_tri(rng, n, lower) for _ in range(batch)])
    A = rng.standard_normal((batch, m, n) if rightside else (batch, n, m))
    Bbar = rng.standard_normal(A.shape)
    junk = Ts.copy()
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    junk[:, other[0], other[1]] = np.nan
    for fn in (orc.trmm_backward, orc.trsm_backward):
        a0, l0 = fn(Ts, A, Bbar, lower=lower, trans=trans, rightside=rightside, alpha=0.5)
        a1, l1 = fn(junk, A, Bbar, lower=lower, trans=trans, rightside=rightside, alpha=0.5)
        assert np.array_equal(a0, a1) and np.array_equal(l0, l1)
        for b in range(batch):  # batch items are independent
            ab, lb = fn(Ts[b], A[b], Bbar[b], lower=lower, trans=trans, rightside=rightside, alpha=0.5)
            assert np.array_equal(ab, a0[b]) and np.array_equal(lb, l0[b])


@pytest.mark.parametrize("trans", [False, True])
@pytest.mark.parametrize("n,k", [(1, 1), (4, 6), (9, 3)])
def test_syrk_backward(orc, trans, n, k):
    rng = np.random.default_rng(500 + n + k)
    A = rng.standard_normal((k, n) if trans else (n, k))
    Bbar = rng.standard_normal((n, n))  # not symmetric on purpose
    alpha = -0.6
    fwd = (lambda a: alpha * a.T @ a) if trans else (lambda a: alpha * a @ a.T)
    g = np.zeros_like(A)
    h = 1e-6
    for idx in np.ndindex(*A.shape):
        Ap, Am = A.copy(), A.copy()
        Ap[idx] += h
        Am[idx] -= h
        g[idx] = (np.sum(Bbar * fwd(Ap)) - np.sum(Bbar * fwd(Am))) / (2 * h)
    S = Bbar + Bbar.T
    closed = alpha * (A @ S) if trans else alpha * (S @ A)
    Abar = orc.syrk_backward(A, Bbar, trans=trans, alpha=alpha)
    assert relerr(Abar, closed) < 1e-13
    assert relerr(Abar, g) < 1e-7


def test_backward_ops_empty(orc):
    z = np.zeros((0, 3, 3))
    a, l = orc.trsm_backward(z, np.zeros((0, 3, 2)), np.zeros((0, 3, 2)))
    assert a.shape == (0, 3, 2) and l.shape == (0, 3, 3)
    assert orc.syrk_backward(np.zeros((2, 0, 4)), np.zeros((2, 0, 0))).shape == (2, 0, 4)


# ----------------------------------------------------------------------------
# gemm2 backward, potri forward / backward
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("m,n,k", [(1, 1, 1), (3, 5, 4), (6, 2, 7)])
def test_gemm2_backward(orc, ta, tb, m, n, k):
    rng = np.random.default_rng(600 + m + 10 * n + 100 * k)
    A = rng.standard_normal((k, m) if ta else (m, k))
    B = rng.standard_normal((n, k) if tb else (k, n))
    Cbar = rng.standard_normal((m, n))
    alpha = 1.3
    fwd = lambda a, b: alpha * (a.T if ta else a) @ (b.T if tb else b)
    h = 1e-6
    gA, gB = np.zeros_like(A), np.zeros_like(B)
    for idx in np.ndindex(*A.shape):
        Ap, Am = A.copy(), A.copy()
        Ap[idx] += h
        Am[idx] -= h
        gA[idx] = (np.sum(Cbar * fwd(Ap, B)) - np.sum(Cbar * fwd(Am, B))) / (2 * h)
    for idx in np.ndindex(*B.shape):
        Bp, Bm = B.copy(), B.copy()
        Bp[idx] += h
        Bm[idx] -= h
        gB[idx] = (np.sum(Cbar * fwd(A, Bp)) - np.sum(Cbar * fwd(A, Bm))) / (2 * h)
    Abar, Bbar = orc.gemm2_backward(A, B, Cbar, ta=ta, tb=tb, alpha=alpha)
    assert relerr(Abar, gA) < 1e-7 and relerr(Bbar, gB) < 1e-7
    # the printed rule: each gradient is itself a gemm2 of Cbar with the other operand
    tB = B.T if tb else B
    tA = A.T if ta else A
    cA = alpha * (tB @ Cbar.T if ta else Cbar @ tB.T)
    cB = alpha * (Cbar.T @ tA if tb else tA.T @ Cbar)
    assert relerr(Abar, cA) < 1e-13 and relerr(Bbar, cB) < 1e-13


@pytest.mark.parametrize("lower", [True, False])
@pytest.mark.parametrize("n", [1, 2, 5, 12, 40])
def test_potri_is_the_inverse(orc, lower, n):
    rng = np.random.default_rng(700 + n)
    X = rng.standard_normal((n, 2 * n))
    A = X @ X.T / (2 * n) + np.eye(n)
    F = np.linalg.cholesky(A)
    F = F if lower else F.T.copy()
    junk = F.copy()
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    junk[other] = np.nan  # the other triangle of the factor is never read
    B = orc.potri(junk, lower=lower)
    assert relerr(B @ A, np.eye(n)) < 1e-12
    assert relerr(B, B.T) < 1e-13
    assert relerr(B, np.linalg.inv(A)) < 1e-12


def test_potri_closed_form(orc):
    # A = [[4, 2], [2, 5]]: L = [[2, 0], [1, 2]], A^-1 = 1/16 [[5, -2], [-2, 4]]
    L = np.array([[2.0, 0.0], [1.0, 2.0]])
    assert np.allclose(orc.potri(L), np.array([[5.0, -2.0], [-2.0, 4.0]]) / 16.0, rtol=0, atol=1e-15)
    assert np.allclose(orc.potri(np.array([[3.0]])), [[1.0 / 9.0]])


@pytest.mark.parametrize("lower", [True, False])
@pytest.mark.parametrize("n", [1, 3, 6])
def test_potri_backward_finite_differences(orc, lower, n):
    rng = np.random.default_rng(800 + n)
    F = rand_tri(rng, n, lower)
    Bbar = rng.standard_normal((n, n))  # not symmetric
    inv_of = (lambda f: np.linalg.inv(f @ f.T)) if lower else (lambda f: np.linalg.inv(f.T @ f))
    g = np.zeros_like(F)
    h = 1e-6
    for i in range(n):
        for j in range(n):
            if (i >= j) if lower else (i <= j):
                Fp, Fm = F.copy(), F.copy()
                Fp[i, j] += h
                Fm[i, j] -= h
                g[i, j] = (np.sum(Bbar * inv_of(Fp)) - np.sum(Bbar * inv_of(Fm))) / (2 * h)
    B = inv_of(F)
    Lbar = orc.potri_backward(F, B, Bbar, lower=lower)
    assert relerr(Lbar, g) < 1e-6
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    assert np.all(Lbar[other] == 0.0)
    # the printed expressions with dense inverses
    S = 0.5 * (Bbar + Bbar.T)
    Fi = np.linalg.inv(F)
    closed = -2 * np.tril(B @ S @ Fi.T) if lower else -2 * np.triu(Fi.T @ S @ B)
    assert relerr(Lbar, closed) < 1e-12
