"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and assembles input matrices (SPD matrices,
right-hand sides, upstream gradients).  It holds none of the arithmetic of the
operators under test and is the one module both the HIP tests/benchmarks and the
CPU oracle's tests may share.

Every draw is numpy ``default_rng(seed)`` with ``seed = SEED0 + 1000*config + tensor``,
made in fp64 and then cast to the configuration's dtype, so the oracle (which widens
fp32 to fp64 exactly) and the GPU see the same bytes.

The inputs stand in for the paper's workloads: batch mode over many small matrices
(section 4.1), the Gaussian-process criterion of section 3.1, and the size sweep of
the Cholesky runtime figure in section 6.
"""
from dataclasses import dataclass

import numpy as np

SEED0 = 171008717


def _rng(config, tensor):
    return np.random.default_rng(SEED0 + 1000 * config + tensor)


@dataclass
class Config:
    name: str
    index: int
    batch: int
    n: int
    dtype: str  # "f32" | "f64"
    m: int = 0  # right-hand sides (0: none)
    note: str = ""


CONFIGS = {
    "C1": Config("C1", 1, 16, 32, "f64", 8, "parity reference: potrf, trsm(8 rhs), sumlogdiag, backward"),
    "C2": Config("C2", 2, 65536, 16, "f32", 0, "tiny-matrix throughput: potrf + backward"),
    "C3": Config("C3", 3, 256, 128, "f32", 1, "GP marginal likelihood: potrf, 2 trsm, sumlogdiag, backward"),
    "C4": Config("C4", 4, 32, 512, "f64", 64, "medium blocked: potrf, trsm, trmm, backward"),
    "C5": Config("C5", 5, 1, 8192, "f64", 512, "large single: potrf, trsm, backward (also f32)"),
}


def np_dtype(dtype):
    return {"f32": np.float32, "f64": np.float64}[dtype]


def spd_wishart(config, batch, n, k, shift, dtype, tensor=0):
    """A = X X^T / k + shift * I with X (n x k) iid N(0,1); symmetric by construction."""
    rng = _rng(config, tensor)
    A = np.empty((batch, n, n), dtype=np.float64)
    # generate in slabs so the X draw never holds more than ~1 GiB
    slab = max(1, min(batch, (1 << 27) // max(1, n * k)))
    for b0 in range(0, batch, slab):
        b1 = min(batch, b0 + slab)
        X = rng.standard_normal((b1 - b0, n, k))
        A[b0:b1] = X @ X.transpose(0, 2, 1)
    A /= k
    idx = np.arange(n)
    A[:, idx, idx] += shift
    A = 0.5 * (A + A.transpose(0, 2, 1))
    return A.astype(np_dtype(dtype))


def lower_normal(config, batch, n, dtype, tensor=1):
    """Upstream gradient Lbar: lower-triangular iid N(0,1), zeros above the diagonal."""
    rng = _rng(config, tensor)
    return np.tril(rng.standard_normal((batch, n, n))).astype(np_dtype(dtype))


def rhs_normal(config, batch, rows, cols, dtype, tensor=2):
    rng = _rng(config, tensor)
    return rng.standard_normal((batch, rows, cols)).astype(np_dtype(dtype))


def rbf_kernel(config, batch, n, dims, lengthscale, variance, jitter, dtype, tensor=0):
    """A_ij = variance * exp(-|p_i - p_j|^2 / (2 l^2)) + jitter * delta_ij, points ~ U[-2,2]^dims."""
    rng = _rng(config, tensor)
    P = rng.uniform(-2.0, 2.0, size=(batch, n, dims))
    sq = np.sum(P * P, axis=-1)
    d2 = sq[:, :, None] + sq[:, None, :] - 2.0 * (P @ P.transpose(0, 2, 1))
    np.maximum(d2, 0.0, out=d2)
    A = variance * np.exp(-0.5 * d2 / (lengthscale * lengthscale))
    idx = np.arange(n)
    A[:, idx, idx] = variance + jitter
    A = 0.5 * (A + A.transpose(0, 2, 1))
    return A.astype(np_dtype(dtype))


def make(name, batch=None, n=None, dtype=None, m=None, lengthscale=1.0, jitter=1e-2):
    """Inputs of configuration ``name`` (optionally shrunk for tests: batch / n / m / dtype).

    Returns a dict of numpy arrays: always ``A`` and ``Lbar``; ``rhs`` where the
    configuration has right-hand sides; ``y`` for the GP configuration.
    """
    c = CONFIGS[name]
    batch = c.batch if batch is None else batch
    n = c.n if n is None else n
    dtype = c.dtype if dtype is None else dtype
    m = c.m if m is None else m
    out = {"config": c, "batch": batch, "n": n, "dtype": dtype, "m": m}
    if name == "C1":
        out["A"] = spd_wishart(1, batch, n, 2 * n, 1.0, dtype)
    elif name == "C2":
        out["A"] = spd_wishart(2, batch, n, 2 * n, 0.5, dtype)
    elif name == "C3":
        out["A"] = rbf_kernel(3, batch, n, 8, lengthscale, 1.0, jitter, dtype)
        out["y"] = rhs_normal(3, batch, n, 1, dtype)[..., 0]
    elif name == "C4":
        out["A"] = spd_wishart(4, batch, n, 2 * n, 1.0, dtype)
    elif name == "C5":
        out["A"] = spd_wishart(5, batch, n, 2 * n, 1.0, dtype)
    else:
        raise KeyError(name)
    out["Lbar"] = lower_normal(c.index, batch, n, dtype)
    if m and name != "C3":
        out["rhs"] = rhs_normal(c.index, batch, n, m, dtype)
    return out


def make_sgp(U, n, dims=4, dtype="f64", lengthscale=1.0, jitter=0.1, noise_var=0.1):
    """Synthetic inputs of the sparse-GP criterion (section 3.2) with the shape of the paper's
    "power" experiment (n = 9568 cases of input dimension four, U inducing points): inputs and
    inducing points ~ U[-2, 2]^dims, RBF kernel of unit variance, Kuu with ``jitter`` on its
    diagonal (which keeps cond(Kuu) within a few hundred), targets ~ N(0, 1)."""
    rng = np.random.default_rng(SEED0 + 9000 + U + n)
    X = rng.uniform(-2.0, 2.0, size=(n, dims))
    Z = rng.uniform(-2.0, 2.0, size=(U, dims))

    def k(a, b):
        d2 = np.sum(a * a, axis=1)[:, None] + np.sum(b * b, axis=1)[None, :] - 2.0 * (a @ b.T)
        return np.exp(-0.5 * np.maximum(d2, 0.0) / (lengthscale * lengthscale))

    Kuu = k(Z, Z)
    Kuu = 0.5 * (Kuu + Kuu.T) + jitter * np.eye(U)
    dt = np_dtype(dtype)
    return {"U": U, "n": n, "dtype": dtype, "Kuu": Kuu.astype(dt), "Kuf": k(Z, X).astype(dt),
            "Kff_diag": np.ones(n, dtype=dt), "y": rng.standard_normal(n).astype(dt), "noise_var": float(noise_var)}


def make_kalman(batch, T, dh, dv, dtype="f32", shared=True, seed=0):
    """Synthetic inputs of the Kalman filter (section 3.4): a Gaussian linear dynamical system
    with a stable transition matrix (0.9 times a random rotation plus a small perturbation),
    an emission matrix ~ N(0, 1/dh), covariances W W^T / (2 d) + c I (c = 0.05 for the state
    noise, 0.2 for the observation noise, 1 for the prior), mu_0 ~ N(0, 1), and observations
    drawn from that very model -- the use the section describes is fitting one model to many
    time series, so the parameters are shared by default; ``shared=False`` draws one set per
    sequence."""
    rng = np.random.default_rng(SEED0 + 7000 + 131 * dh + 17 * dv + seed)
    pb = 1 if shared else batch

    def spd(d, c):
        W = rng.standard_normal((pb, d, 2 * d))
        return W @ W.transpose(0, 2, 1) / (4.0 * d) + c * np.eye(d)

    Q, _ = np.linalg.qr(rng.standard_normal((pb, dh, dh)))
    A = 0.9 * Q + 0.02 * rng.standard_normal((pb, dh, dh))
    B = rng.standard_normal((pb, dv, dh)) / np.sqrt(dh)
    Sh, Sv, S0 = spd(dh, 0.05), spd(dv, 0.2), spd(dh, 1.0)
    mu0 = rng.standard_normal((pb, dh))
    # simulate
    ch, cv, c0 = np.linalg.cholesky(Sh), np.linalg.cholesky(Sv), np.linalg.cholesky(S0)
    h = mu0 + np.einsum("bij,bj->bi", c0, rng.standard_normal((batch, dh)))
    v = np.empty((batch, T, dv))
    for t in range(T):
        if t > 0:
            h = np.einsum("bij,bj->bi", A, h) + np.einsum("bij,bj->bi", ch, rng.standard_normal((batch, dh)))
        v[:, t] = np.einsum("bij,bj->bi", B, h) + np.einsum("bij,bj->bi", cv, rng.standard_normal((batch, dv)))
    dt = np_dtype(dtype)
    sq = (lambda x: x[0]) if shared else (lambda x: x)
    return {"batch": batch, "T": T, "dh": dh, "dv": dv, "dtype": dtype, "shared": shared,
            "A": sq(A).astype(dt), "B": sq(B).astype(dt), "Sh": sq(Sh).astype(dt), "Sv": sq(Sv).astype(dt),
            "mu0": sq(mu0).astype(dt), "S0": sq(S0).astype(dt), "v": v.astype(dt)}


def cond_estimate(A, sample=4):
    """2-norm condition numbers of the first ``sample`` matrices (eigvalsh, fp64)."""
    A = np.asarray(A, dtype=np.float64).reshape(-1, A.shape[-2], A.shape[-1])[:sample]
    w = np.linalg.eigvalsh(A)
    return w[:, -1] / w[:, 0]
