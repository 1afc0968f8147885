"""Pins for the CPU oracle: everything here checks ``oracle/`` against something that
is NOT the oracle -- closed forms, brute-force determinants and inverses written in
this file, numpy/scipy routines as a third opinion, finite differences and exact
identities from the paper's appendix.  No GPU needed.
"""
import itertools
import math
import os

import numpy as np
import pytest

import workloads

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
FLAGS = list(itertools.product([True, False], [False, True], [False, True]))  # lower, trans, rightside


# ----------------------------------------------------------------------------
# independent helpers (plain python / numpy, no oracle code)
# ----------------------------------------------------------------------------
def det_leibniz(A):
    n = A.shape[0]
    total = 0.0
    for perm in itertools.permutations(range(n)):
        inv = sum(1 for i in range(n) for j in range(i + 1, n) if perm[i] > perm[j])
        p = 1.0
        for i in range(n):
            p *= A[i, perm[i]]
        total += -p if inv % 2 else p
    return total


def logdet_lu(A):
    """log|det A| by Gaussian elimination with partial pivoting, python loops."""
    M = np.array(A, dtype=np.float64)
    n = M.shape[0]
    s = 0.0
    for k in range(n):
        p = k + int(np.argmax(np.abs(M[k:, k])))
        if p != k:
            M[[k, p]] = M[[p, k]]
        s += math.log(abs(M[k, k]))
        for i in range(k + 1, n):
            f = M[i, k] / M[k, k]
            M[i, k:] -= f * M[k, k:]
    return s


def inverse_gauss_jordan(A):
    n = A.shape[0]
    M = np.hstack([np.array(A, dtype=np.float64), np.eye(n)])
    for k in range(n):
        p = k + int(np.argmax(np.abs(M[k:, k])))
        if p != k:
            M[[k, p]] = M[[p, k]]
        M[k] /= M[k, k]
        for i in range(n):
            if i != k:
                M[i] -= M[i, k] * M[k]
    return M[:, n:]


def rand_spd(rng, n, batch=None):
    shape = (n, 2 * n) if batch is None else (batch, n, 2 * n)
    X = rng.standard_normal(shape)
    A = X @ np.swapaxes(X, -1, -2) / (2 * n) + np.eye(n)
    return 0.5 * (A + np.swapaxes(A, -1, -2))


def rand_tri(rng, n, lower, batch=None):
    shape = (n, n) if batch is None else (batch, n, n)
    T = rng.standard_normal(shape) * 0.3
    T = np.tril(T) if lower else np.triu(T)
    idx = np.arange(n)
    T[..., idx, idx] = 1.0 + rng.uniform(0.0, 1.0, size=shape[:-1])
    return T


def op(T, trans):
    return np.swapaxes(T, -1, -2) if trans else T


def relerr(x, ref):
    return np.linalg.norm(np.asarray(x) - ref) / max(np.linalg.norm(ref), 1e-300)


def load_golden(name):
    return np.loadtxt(os.path.join(GOLD, name), comments="#")


# ----------------------------------------------------------------------------
# potrf forward
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("n", [1, 2, 3, 7, 16, 33, 64, 100])
def test_potrf_reconstructs_and_is_lower(orc, n):
    rng = np.random.default_rng(n)
    A = rand_spd(rng, n, batch=3)
    L, info = orc.potrf(A, return_info=True)
    assert np.all(info == 0)
    assert np.all(np.triu(L, 1) == 0.0)  # exact zeros above the diagonal
    assert np.all(np.diagonal(L, axis1=-2, axis2=-1) > 0)
    assert relerr(L @ L.transpose(0, 2, 1), A) < 1e-14 * max(n, 4)


def test_potrf_2x2_closed_form(orc):
    a, b, c = 4.0, 1.2, 3.0
    L = orc.potrf(np.array([[a, b], [b, c]]))
    ref = np.array([[math.sqrt(a), 0.0], [b / math.sqrt(a), math.sqrt(c - b * b / a)]])
    assert np.allclose(L, ref, rtol=1e-15, atol=0)


def test_potrf_minij_is_all_ones(orc):
    n = 12
    i = np.arange(1, n + 1)
    A = np.minimum.outer(i, i).astype(np.float64)
    L = orc.potrf(A)
    assert np.array_equal(L, np.tril(np.ones((n, n))))  # exact in floating point


def test_potrf_pascal_golden(orc):
    Lref = load_golden("pascal_lower_n8.txt")
    n = Lref.shape[0]
    S = np.array([[math.comb(i + j, i) for j in range(n)] for i in range(n)], dtype=np.float64)
    L = orc.potrf(S)
    assert np.allclose(L, Lref, rtol=1e-12, atol=1e-12)
    R = orc.potrf(S, lower=False)
    assert np.allclose(R, Lref.T, rtol=1e-12, atol=1e-12)


def test_potrf_tridiagonal_golden(orc):
    Lref = load_golden("tridiag_factor_n8.txt")
    n = Lref.shape[0]
    T = 2 * np.eye(n) - np.eye(n, k=1) - np.eye(n, k=-1)
    assert np.allclose(orc.potrf(T), Lref, rtol=1e-14, atol=1e-15)


def test_potrf_diagonal_and_scalar(orc):
    d = np.array([4.0, 9.0, 0.25, 16.0])
    assert np.array_equal(orc.potrf(np.diag(d)), np.diag(np.sqrt(d)))
    assert np.array_equal(orc.potrf(np.array([[2.25]])), np.array([[1.5]]))


@pytest.mark.parametrize("n", [5, 40])
def test_potrf_matches_numpy_cholesky(orc, n):
    A = rand_spd(np.random.default_rng(7 + n), n, batch=4)
    assert relerr(orc.potrf(A), np.linalg.cholesky(A)) < 1e-13


@pytest.mark.parametrize("n", [1, 4, 9, 31])
def test_potrf_upper_is_transpose_of_lower(orc, n):
    A = rand_spd(np.random.default_rng(n + 100), n, batch=2)
    L = orc.potrf(A, lower=True)
    R = orc.potrf(A, lower=False)
    assert np.all(np.tril(R, -1) == 0.0)
    assert relerr(R, L.transpose(0, 2, 1)) < 1e-14
    assert relerr(R.transpose(0, 2, 1) @ R, A) < 1e-13


def test_potrf_reads_only_its_triangle(orc):
    rng = np.random.default_rng(5)
    n = 9
    A = rand_spd(rng, n)
    Al = A.copy()
    Al[np.triu_indices(n, 1)] = np.nan  # junk above: lower variant must ignore it
    Au = A.copy()
    Au[np.tril_indices(n, -1)] = np.nan
    assert np.array_equal(orc.potrf(Al, lower=True), orc.potrf(A, lower=True))
    assert np.array_equal(orc.potrf(Au, lower=False), orc.potrf(A, lower=False))


def test_potrf_info_reports_first_bad_pivot(orc):
    n = 6
    A = np.eye(n)
    A[3, 3] = -1.0  # pivot 4 (1-based) is not positive
    B = rand_spd(np.random.default_rng(2), n)
    L, info = orc.potrf(np.stack([B, A, B]), return_info=True)
    assert list(info) == [0, 4, 0]
    assert relerr(L[0] @ L[0].T, B) < 1e-14
    Z = np.zeros((2, 2))
    assert list(orc.potrf(Z, return_info=True)[1]) == [1]
    _, info_u = orc.potrf(np.stack([B, A]), lower=False, return_info=True)
    assert list(info_u) == [0, 4]


def test_potrf_in_place(orc):
    A = rand_spd(np.random.default_rng(11), 13, batch=3)
    ref = orc.potrf(A)
    work = A.copy()
    orc.potrf_inplace(work)
    assert np.array_equal(work, ref)


def test_potrf_empty(orc):
    assert orc.potrf(np.zeros((0, 4, 4))).shape == (0, 4, 4)
    assert orc.potrf(np.zeros((3, 0, 0))).shape == (3, 0, 0)


# ----------------------------------------------------------------------------
# sumlogdiag
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("n", [1, 2, 4, 6])
def test_sumlogdiag_is_half_logdet_leibniz(orc, n):
    A = rand_spd(np.random.default_rng(n), n)
    s = orc.sumlogdiag(orc.potrf(A))
    assert abs(float(s) - 0.5 * math.log(det_leibniz(A))) < 1e-13 * max(1, n)


@pytest.mark.parametrize("n", [10, 50])
def test_sumlogdiag_is_half_logdet_lu(orc, n):
    A = rand_spd(np.random.default_rng(n), n, batch=3)
    s = orc.sumlogdiag(orc.potrf(A))
    ref = np.array([0.5 * logdet_lu(a) for a in A])
    assert np.allclose(s, ref, rtol=1e-12, atol=1e-12)


def test_sumlogdiag_plain_log(orc):
    L = np.diag([math.e, math.e ** 2, 1.0])
    assert abs(float(orc.sumlogdiag(L)) - 3.0) < 1e-15
    L[0, 2] = 77.0  # off-diagonal entries play no part
    assert abs(float(orc.sumlogdiag(L)) - 3.0) < 1e-15
    assert np.isnan(orc.sumlogdiag(np.diag([1.0, -1.0])))  # no abs(), IEEE semantics


# ----------------------------------------------------------------------------
# trsm / trmm
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("n,m", [(1, 1), (3, 5), (8, 2), (17, 9)])
def test_trsm_against_dense_inverse(orc, lower, trans, rightside, n, m):
    rng = np.random.default_rng(1000 + n * 10 + m)
    T = rand_tri(rng, n, lower)
    A = rng.standard_normal((m, n) if rightside else (n, m))
    alpha = 0.75
    Tinv = inverse_gauss_jordan(op(T, trans))
    ref = alpha * (A @ Tinv if rightside else Tinv @ A)
    B = orc.trsm(T, A, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    assert relerr(B, ref) < 1e-12
    # residual against the definition t(L) B = alpha A (or B t(L) = alpha A)
    back = B @ op(T, trans) if rightside else op(T, trans) @ B
    assert relerr(back, alpha * A) < 1e-13


@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
def test_trsm_ignores_other_triangle_and_inplace(orc, lower, trans, rightside):
    rng = np.random.default_rng(3)
    n, m = 7, 4
    T = rand_tri(rng, n, lower, batch=2)
    junk = T.copy()
    mask = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    junk[:, mask[0], mask[1]] = np.nan
    A = rng.standard_normal((2, m, n) if rightside else (2, n, m))
    ref = orc.trsm(T, A, lower=lower, trans=trans, rightside=rightside)
    assert np.array_equal(orc.trsm(junk, A, lower=lower, trans=trans, rightside=rightside), ref)
    work = A.copy()
    orc.trsm(T, work, lower=lower, trans=trans, rightside=rightside, inplace=True)
    assert np.array_equal(work, ref)
    # scipy as a third opinion
    from scipy.linalg import solve_triangular

    for b in range(2):
        if rightside:  # X t(T) = A  <=>  t(T)^T X^T = A^T
            x = solve_triangular(T[b], A[b].T, lower=lower, trans=0 if trans else 1).T
        else:
            x = solve_triangular(T[b], A[b], lower=lower, trans=1 if trans else 0)
        assert relerr(ref[b], x) < 1e-13


def test_trsm_identity_and_diagonal(orc):
    rng = np.random.default_rng(4)
    A = rng.standard_normal((5, 3))
    assert np.array_equal(orc.trsm(np.eye(5), A, alpha=2.0), 2.0 * A)
    d = np.array([1.0, 2.0, 4.0, 8.0, 0.5])
    assert np.allclose(orc.trsm(np.diag(d), A), A / d[:, None], rtol=1e-15)
    assert np.allclose(orc.trsm(np.diag(d), A.T.copy(), rightside=True), A.T / d[None, :], rtol=1e-15)


@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("n,m", [(1, 2), (6, 3), (19, 8)])
def test_trmm_against_dense_product(orc, lower, trans, rightside, n, m):
    rng = np.random.default_rng(2000 + n + m)
    T = rand_tri(rng, n, lower, batch=2)
    junk = T.copy()
    mask = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    junk[:, mask[0], mask[1]] = np.nan
    A = rng.standard_normal((2, m, n) if rightside else (2, n, m))
    alpha = -1.5
    ref = alpha * (A @ op(T, trans) if rightside else op(T, trans) @ A)
    B = orc.trmm(junk, A, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    assert relerr(B, ref) < 1e-14
    work = A.copy()
    orc.trmm(T, work, lower=lower, trans=trans, rightside=rightside, alpha=alpha, inplace=True)
    assert np.array_equal(work, B)


@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("n,m,batch", [(96, 40, 2), (380, 400, 1)])
def test_trsm_trmm_larger_sizes_against_scipy_and_dense_product(orc, lower, trans, rightside, n, m, batch):
    """From n = 64 on the right-side operators read t(L) from a copy with the summation index
    contiguous, and one matrix with n * n * m > 5e7 hands its vectors to the threads in chunks:
    both against scipy's triangular solve and numpy's dense product, NaN in the unread triangle."""
    from scipy.linalg import solve_triangular

    rng = np.random.default_rng(7000 + n)
    T = rand_tri(rng, n, lower, batch=batch)
    T[:, np.arange(n), np.arange(n)] = 1.5 + np.abs(T[:, np.arange(n), np.arange(n)])  # keep the solves tame
    T[:, np.tril_indices(n, -1)[0], np.tril_indices(n, -1)[1]] *= 0.1
    T[:, np.triu_indices(n, 1)[0], np.triu_indices(n, 1)[1]] *= 0.1
    junk = T.copy()
    mask = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    junk[:, mask[0], mask[1]] = np.nan
    A = rng.standard_normal((batch, m, n) if rightside else (batch, n, m))
    X = orc.trsm(junk, A, lower=lower, trans=trans, rightside=rightside, alpha=0.5)
    P = orc.trmm(junk, A, lower=lower, trans=trans, rightside=rightside, alpha=0.5)
    for b in range(batch):
        if rightside:
            x = solve_triangular(T[b], 0.5 * A[b].T, lower=lower, trans=0 if trans else 1).T
            pr = 0.5 * A[b] @ op(T[b], trans)
        else:
            x = solve_triangular(T[b], 0.5 * A[b], lower=lower, trans=1 if trans else 0)
            pr = 0.5 * op(T[b], trans) @ A[b]
        assert relerr(X[b], x) < 1e-12
        assert relerr(P[b], pr) < 1e-13


@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
def test_trmm_undoes_trsm(orc, lower, trans, rightside):
    rng = np.random.default_rng(6)
    n, m = 24, 5
    T = rand_tri(rng, n, lower)
    A = rng.standard_normal((m, n) if rightside else (n, m))
    B = orc.trsm(T, A, lower=lower, trans=trans, rightside=rightside)
    assert relerr(orc.trmm(T, B, lower=lower, trans=trans, rightside=rightside), A) < 1e-13


# ----------------------------------------------------------------------------
# syrk
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("trans", [False, True])
@pytest.mark.parametrize("n,k", [(1, 1), (4, 9), (13, 5)])
def test_syrk_against_numpy(orc, trans, n, k):
    rng = np.random.default_rng(n * 7 + k)
    A = rng.standard_normal((3, k, n) if trans else (3, n, k))
    alpha = 0.3
    ref = alpha * (A.transpose(0, 2, 1) @ A if trans else A @ A.transpose(0, 2, 1))
    B = orc.syrk(A, trans=trans, alpha=alpha)
    assert relerr(B, ref) < 1e-14
    assert np.array_equal(B, B.transpose(0, 2, 1))  # exactly symmetric, both triangles written


def test_syrk_of_factor_gives_back_matrix(orc):
    A = rand_spd(np.random.default_rng(8), 21, batch=2)
    L = orc.potrf(A)
    assert relerr(orc.syrk(L), A) < 1e-14
    R = orc.potrf(A, lower=False)
    assert relerr(orc.syrk(R, trans=True), A) < 1e-14


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("m,n,k", [(1, 1, 1), (3, 5, 4), (7, 2, 9)])
def test_gemm2_against_numpy(orc, ta, tb, m, n, k):
    rng = np.random.default_rng(m * 100 + n * 10 + k)
    A = rng.standard_normal((2, k, m) if ta else (2, m, k))
    B = rng.standard_normal((2, n, k) if tb else (2, k, n))
    ref = -0.5 * (op(A, ta) @ op(B, tb))
    assert relerr(orc.gemm2(A, B, ta=ta, tb=tb, alpha=-0.5), ref) < 1e-14


# ----------------------------------------------------------------------------
# potrf backward
# ----------------------------------------------------------------------------
def fd_potrf_grad(A, Lbar, h=1e-6, lower=True):
    """Central differences of phi(A) = <Lbar, chol(A)> along symmetric directions.
    E = e_i e_j^T + e_j e_i^T gives 2 Abar_ij, E = e_i e_i^T gives Abar_ii."""
    n = A.shape[0]
    G = np.zeros((n, n))

    def phi(M):
        C = np.linalg.cholesky(M)
        return float(np.sum(Lbar * (C if lower else C.T)))

    for i in range(n):
        for j in range(i + 1):
            E = np.zeros((n, n))
            E[i, j] = 1.0
            E[j, i] = 1.0
            d = (phi(A + h * E) - phi(A - h * E)) / (2 * h)
            G[i, j] = G[j, i] = d if i == j else 0.5 * d
    return G


@pytest.mark.parametrize("n", [1, 2, 5, 8])
def test_backward_against_finite_differences(orc, n):
    rng = np.random.default_rng(30 + n)
    A = rand_spd(rng, n)
    Lbar = np.tril(rng.standard_normal((n, n)))
    L = orc.potrf(A)
    Abar = orc.potrf_backward(L, Lbar)
    assert relerr(Abar, fd_potrf_grad(A, Lbar)) < 2e-8
    # upper factor
    Rbar = np.triu(rng.standard_normal((n, n)))
    Abar_u = orc.potrf_backward(orc.potrf(A, lower=False), Rbar, lower=False)
    assert relerr(Abar_u, fd_potrf_grad(A, Rbar, lower=False)) < 2e-8


@pytest.mark.parametrize("n", [1, 3, 10, 37])
def test_backward_closed_forms(orc, n):
    rng = np.random.default_rng(40 + n)
    A = rand_spd(rng, n)
    L = orc.potrf(A)
    # phi = <L, L>/2 = tr(A)/2  =>  Abar = I/2   (Lbar = L)
    assert np.allclose(orc.potrf_backward(L, L), 0.5 * np.eye(n), rtol=0, atol=1e-13)
    # phi = sum log l_ii = logdet(A)/2  =>  Abar = inv(A)/2   (Lbar = diag(1/l_ii))
    Abar = orc.potrf_backward(L, np.diag(1.0 / np.diag(L)))
    assert relerr(Abar, 0.5 * inverse_gauss_jordan(A)) < 1e-12
    # zero upstream gradient
    assert np.array_equal(orc.potrf_backward(L, np.zeros((n, n))), np.zeros((n, n)))


def test_backward_scalar(orc):
    a, g = 7.0, 3.0
    out = orc.potrf_backward(np.array([[math.sqrt(a)]]), np.array([[g]]))
    assert abs(out[0, 0] - g / (2 * math.sqrt(a))) < 1e-15


@pytest.mark.parametrize("n", [4, 12, 30])
def test_backward_adjoint_identity(orc, n):
    """<Lbar, dL> = <Abar, dA> with dL = 1/2 L (L^-1 dA L^-T o E), appendix (potrf)."""
    rng = np.random.default_rng(50 + n)
    A = rand_spd(rng, n)
    L = np.linalg.cholesky(A)
    Lbar = np.tril(rng.standard_normal((n, n)))
    dA = rng.standard_normal((n, n))
    dA = dA + dA.T
    E = np.tril(2 * np.ones((n, n)), -1) + np.eye(n)
    Li = inverse_gauss_jordan(L)
    dL = 0.5 * L @ ((Li @ dA @ Li.T) * E)
    Abar = orc.potrf_backward(orc.potrf(A), Lbar)
    lhs = float(np.sum(Lbar * dL))
    rhs = float(np.sum(Abar * dA))
    assert abs(lhs - rhs) < 1e-11 * max(1.0, abs(lhs))


@pytest.mark.parametrize("n", [3, 9, 26])
def test_backward_structure(orc, n):
    rng = np.random.default_rng(60 + n)
    A = rand_spd(rng, n, batch=2)
    L = orc.potrf(A)
    Lbar = np.tril(rng.standard_normal((2, n, n)))
    Abar = orc.potrf_backward(L, Lbar)
    assert relerr(Abar, Abar.transpose(0, 2, 1)) < 1e-13  # symmetric
    # independent of whatever sits above the diagonal of L and Lbar
    up = np.triu_indices(n, 1)
    Lj, Gj = L.copy(), Lbar.copy()
    Lj[:, up[0], up[1]] = 1e6 * rng.standard_normal(len(up[0]))
    Gj[:, up[0], up[1]] = 1e6 * rng.standard_normal(len(up[0]))
    assert relerr(orc.potrf_backward(Lj, Gj), Abar) < 1e-13
    # linear in Lbar
    G2 = np.tril(rng.standard_normal((2, n, n)))
    lin = orc.potrf_backward(L, 2.0 * Lbar - 3.0 * G2)
    assert relerr(lin, 2.0 * Abar - 3.0 * orc.potrf_backward(L, G2)) < 1e-12
    # the two independently coded orders agree: copyltu-first vs Phi-then-sym
    assert relerr(orc.potrf_backward_phi(L, Lbar), Abar) < 1e-12
    # aliasing Abar == Lbar
    work = Lbar.copy()
    orc.potrf_backward(L, work, inplace=True)
    assert np.array_equal(work, Abar)


@pytest.mark.parametrize("n", [2, 7, 20])
def test_backward_upper_matches_lower_on_transposes(orc, n):
    rng = np.random.default_rng(70 + n)
    A = rand_spd(rng, n)
    R = orc.potrf(A, lower=False)
    Rbar = np.triu(rng.standard_normal((n, n)))
    up = orc.potrf_backward(R, Rbar, lower=False)
    lo = orc.potrf_backward(R.T.copy(), Rbar.T.copy(), lower=True)
    assert relerr(up, lo) < 1e-13


def test_backward_dense_formula_third_opinion(orc):
    """Abar = 1/2 L^-T copyltu(L^T Lbar) L^-1 evaluated with dense numpy algebra."""
    rng = np.random.default_rng(80)
    n = 15
    A = rand_spd(rng, n)
    L = np.linalg.cholesky(A)
    Lbar = np.tril(rng.standard_normal((n, n)))
    P = L.T @ Lbar
    P = np.tril(P) + np.tril(P, -1).T
    Li = inverse_gauss_jordan(L)
    ref = 0.5 * Li.T @ P @ Li
    assert relerr(orc.potrf_backward(orc.potrf(A), Lbar), ref) < 1e-12


# ----------------------------------------------------------------------------
# GP criterion glue
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("n", [3, 12])
def test_gp_loss_and_gradient_closed_form(orc, n):
    """d/dA [1/2 y^T A^-1 y + 1/2 logdet A] = 1/2 (A^-1 - alpha alpha^T), alpha = A^-1 y."""
    rng = np.random.default_rng(90 + n)
    A = rand_spd(rng, n, batch=2)
    y = rng.standard_normal((2, n))
    L = orc.potrf(A)
    z = orc.trsm(L, y[..., None])
    alpha = orc.trsm(L, z, trans=True)
    loss, Lbar = orc.gp_glue(L, y, z[..., 0], alpha[..., 0])
    Abar = orc.potrf_backward(L, Lbar)
    for b in range(2):
        Ai = inverse_gauss_jordan(A[b])
        a = Ai @ y[b]
        ref_loss = 0.5 * float(y[b] @ a) + 0.5 * logdet_lu(A[b])
        assert abs(loss[b] - ref_loss) < 1e-12 * max(1.0, abs(ref_loss))
        assert relerr(Abar[b], 0.5 * (Ai - np.outer(a, a))) < 1e-11
        assert np.all(np.triu(Lbar[b], 1) == 0.0)


# ----------------------------------------------------------------------------
# sampled-entry helpers used by the full-size GPU checks
# ----------------------------------------------------------------------------
def test_entry_helpers(orc):
    rng = np.random.default_rng(99)
    n = 23
    L = np.tril(rng.standard_normal((n, n)))
    X = rng.standard_normal((n, n))
    G = np.tril(rng.standard_normal((n, n)))
    LLt, RtR, LtXL, LtG = L @ L.T, L @ L.T, L.T @ X @ L, L.T @ G
    for (i, j) in [(0, 0), (5, 3), (3, 5), (22, 22), (22, 0), (0, 22), (10, 10)]:
        assert abs(orc.llt_entry(L, i, j) - LLt[i, j]) < 1e-12
        assert abs(orc.llt_entry(L.T.copy(), i, j, lower=False) - RtR[i, j]) < 1e-12
        assert abs(orc.ltxl_entry(L, X, i, j) - LtXL[i, j]) < 1e-11
        assert abs(orc.ltlbar_entry(L, G, i, j) - LtG[i, j]) < 1e-12


# ----------------------------------------------------------------------------
# the synthetic workloads are well conditioned (spec tolerances assume cond <= 1e3)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("name,kw", [
    ("C1", {}), ("C2", {"batch": 64}), ("C3", {"batch": 4}), ("C4", {"batch": 2, "n": 128}),
    ("C5", {"n": 256}), ("C3", {"batch": 2, "lengthscale": 3.0, "jitter": 0.5}),
])
def test_workloads_are_spd_and_well_conditioned(orc, name, kw):
    w = workloads.make(name, **kw)
    A = w["A"]
    assert A.dtype == workloads.np_dtype(w["dtype"])
    assert np.array_equal(A, A.transpose(0, 2, 1))
    assert np.all(workloads.cond_estimate(A) <= 1e3)
    L, info = orc.potrf(A, return_info=True)
    assert np.all(info == 0)
    assert np.all(np.triu(w["Lbar"], 1) == 0)
