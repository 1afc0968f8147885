"""Pins of the oracle's Kalman filter (section 3.4) against things that are not the filter:
the joint Gaussian density of all observations written out densely, the information form of the
measurement update, and the scalar steady state of the Riccati recursion."""
import numpy as np
import pytest

import oracle as orc
import workloads


def joint_gaussian(A, B, Sh, Sv, mu0, S0, T):
    """Mean and covariance of the stacked observations (v_0 .. v_{T-1}) of the linear dynamical
    system, from the model's definition: h_0 ~ N(mu0, S0), h_t = A h_{t-1} + eps_t, v_t = B h_t + xi_t."""
    dh, dv = A.shape[0], B.shape[0]
    means, P = [mu0], [S0]  # marginal mean / covariance of h_t
    for t in range(1, T):
        means.append(A @ means[-1])
        P.append(A @ P[-1] @ A.T + Sh)
    mean = np.concatenate([B @ m for m in means])
    cov = np.zeros((T * dv, T * dv))
    for s in range(T):
        for t in range(s, T):
            C = np.linalg.matrix_power(A, t - s) @ P[s]  # Cov(h_t, h_s)
            blk = B @ C @ B.T
            if s == t:
                blk = blk + Sv
            cov[t * dv:(t + 1) * dv, s * dv:(s + 1) * dv] = blk
            cov[s * dv:(s + 1) * dv, t * dv:(t + 1) * dv] = blk.T
    return mean, cov


@pytest.mark.parametrize("dh,dv,T", [(1, 1, 1), (2, 1, 3), (3, 2, 4), (2, 3, 5), (4, 4, 3)])
def test_nll_is_the_joint_gaussian_density(dh, dv, T):
    w = workloads.make_kalman(3, T, dh, dv, dtype="f64", shared=False, seed=dh + dv + T)
    nll, _, _, info = orc.kalman_filter(w["A"], w["B"], w["Sh"], w["Sv"], w["mu0"], w["S0"], w["v"])
    assert np.all(info == 0)
    for b in range(3):
        mean, cov = joint_gaussian(w["A"][b], w["B"][b], w["Sh"][b], w["Sv"][b], w["mu0"][b], w["S0"][b], T)
        r = w["v"][b].reshape(-1) - mean
        sign, logdet = np.linalg.slogdet(cov)
        ref = 0.5 * (T * dv * np.log(2 * np.pi) + logdet + r @ np.linalg.solve(cov, r))
        assert sign > 0
        assert abs(nll[b] - ref) <= 1e-10 * max(1.0, abs(ref))


def test_measurement_update_equals_information_form():
    dh, dv, T = 4, 3, 6
    w = workloads.make_kalman(2, T, dh, dv, dtype="f64", shared=True, seed=5)
    A, B, Sh, Sv = w["A"], w["B"], w["Sh"], w["Sv"]
    _, f, F, _ = orc.kalman_filter(A, B, Sh, Sv, w["mu0"], w["S0"], w["v"])
    for b in range(2):
        mu_h, S_hh = w["mu0"], w["S0"]
        for t in range(T):
            if t > 0:
                mu_h, S_hh = A @ f[b, t - 1], A @ F[b, t - 1] @ A.T + Sh
            # posterior of h_t given v_t by completing the square
            Pinv = np.linalg.inv(S_hh) + B.T @ np.linalg.inv(Sv) @ B
            Fref = np.linalg.inv(Pinv)
            fref = Fref @ (np.linalg.solve(S_hh, mu_h) + B.T @ np.linalg.solve(Sv, w["v"][b, t]))
            assert np.allclose(F[b, t], Fref, rtol=1e-10, atol=1e-12)
            assert np.allclose(f[b, t], fref, rtol=1e-10, atol=1e-12)
            assert np.allclose(F[b, t], F[b, t].T, rtol=0, atol=1e-14)


def test_scalar_steady_state():
    """dh = dv = 1: F_t -> the positive root of the scalar Riccati fixed point,
    with P = a^2 F + q:  F = P r / (P + r)."""
    a, q, r = 0.8, 0.3, 0.5
    T = 200
    v = np.zeros((1, T, 1))
    _, _, F, _ = orc.kalman_filter(np.array([[a]]), np.array([[1.0]]), np.array([[q]]), np.array([[r]]),
                                   np.array([0.0]), np.array([[2.0]]), v)
    # a^2 F^2 + (q + r - a^2 r) F - q r = 0
    c2, c1, c0 = a * a, q + r - a * a * r, -q * r
    root = (-c1 + np.sqrt(c1 * c1 - 4 * c2 * c0)) / (2 * c2)
    assert abs(F[0, -1, 0, 0] - root) <= 1e-13


def test_shared_parameters_equal_repeated_parameters_and_info():
    w = workloads.make_kalman(4, 5, 3, 2, dtype="f64", shared=True, seed=1)
    rep = {k: np.broadcast_to(w[k], (4,) + w[k].shape).copy() for k in ("A", "B", "Sh", "Sv", "mu0", "S0")}
    a = orc.kalman_filter(w["A"], w["B"], w["Sh"], w["Sv"], w["mu0"], w["S0"], w["v"])
    b = orc.kalman_filter(rep["A"], rep["B"], rep["Sh"], rep["Sv"], rep["mu0"], rep["S0"], w["v"])
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    # an observation covariance that is not positive definite is reported with the step it fails at
    bad = -np.eye(2)
    _, _, _, info = orc.kalman_filter(w["A"], w["B"], w["Sh"], bad * 100.0, w["mu0"], w["S0"], w["v"], want_states=False)
    assert np.all(info == 1)
