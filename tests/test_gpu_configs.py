"""The five benchmark configurations at their full sizes, HIP library vs CPU oracle.

C1-C4 are compared element by element with the oracle on the same seeded inputs.
C5 (one 8192 x 8192 matrix) is too large for the plain-loop oracle to run in full inside a
test, so it is checked (a) element by element on the part of each result that the oracle
can compute alone -- the leading k x k block of the factor and the leading k rows of the
triangular solve depend only on the leading block of the inputs -- (b) on sampled entries
of the defining relations L L^T = A and 2 L^T Abar L = copyltu(L^T Lbar), each entry
evaluated by the oracle, and (c) on the closed form Lbar = L  =>  Abar = I/2, which
involves every tile of the backward pass.  A mid-size single matrix (n = 1024) is compared
in full.
"""
import sys

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

TOL = {"f32": 2e-4, "f64": 1e-10}


@pytest.fixture(scope="module")
def la():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1710_08717_amd as la_mod

    la_mod.load()
    return la_mod


@pytest.fixture(autouse=True)
def _announce(request):
    sys.stderr.write(f"\n[gpu-case] {request.node.nodeid}\n")
    sys.stderr.flush()
    yield


def dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    import torch

    torch.cuda.synchronize()
    return t.cpu().numpy()


def relerr(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if x.ndim < 3:
        x, ref = x[None], ref[None]
    x = x.reshape(x.shape[0], -1)
    ref = ref.reshape(ref.shape[0], -1)
    return float(np.max(np.linalg.norm(x - ref, axis=1) / np.maximum(np.linalg.norm(ref, axis=1), 1e-300)))


def test_c1_reference(la, orc):
    w = workloads.make("C1")
    tol = TOL[w["dtype"]]
    assert np.all(workloads.cond_estimate(w["A"], sample=16) <= 1e3)
    A, G, R = dev(w["A"]), dev(w["Lbar"]), dev(w["rhs"])
    L = la.potrf(A)
    Lr = orc.potrf(w["A"])
    assert relerr(host(L), Lr) <= tol
    assert relerr(host(la.trsm(L, R)), orc.trsm(Lr, w["rhs"])) <= tol
    s = host(la.sumlogdiag(L))
    assert np.max(np.abs(s - orc.sumlogdiag(Lr))) <= tol * np.max(np.abs(orc.sumlogdiag(Lr)))
    assert relerr(host(la.potrf_backward(L, G)), orc.potrf_backward(Lr, w["Lbar"])) <= tol
    # every flag combination of trsm / trmm on this configuration's shapes
    for lower in (True, False):
        T = Lr if lower else np.ascontiguousarray(Lr.transpose(0, 2, 1))
        for trans in (False, True):
            for rightside in (False, True):
                B = w["rhs"].transpose(0, 2, 1).copy() if rightside else w["rhs"]
                kw = dict(lower=lower, trans=trans, rightside=rightside)
                assert relerr(host(la.trsm(dev(T), dev(B), **kw)), orc.trsm(T, B, **kw)) <= tol
                assert relerr(host(la.trmm(dev(T), dev(B), **kw)), orc.trmm(T, B, **kw)) <= tol


def test_c2_tiny_throughput_config(la, orc):
    w = workloads.make("C2")  # 65536 matrices, n = 16, fp32: the launch configuration bench.py times
    tol = TOL[w["dtype"]]
    assert np.all(workloads.cond_estimate(w["A"], sample=64) <= 1e3)
    import torch

    info = torch.zeros(w["batch"], dtype=torch.int32, device="cuda")
    L = la.potrf(dev(w["A"]), info=info)
    Lr = orc.potrf(w["A"])
    assert np.all(host(info) == 0)
    Lh = host(L)
    assert np.all(np.triu(Lh, 1) == 0)
    assert relerr(Lh, Lr) <= tol
    # backward from the GPU's own factor (as in the benchmark) against the oracle on that same factor
    Abar = host(la.potrf_backward(L, dev(w["Lbar"])))
    assert np.array_equal(Abar, Abar.transpose(0, 2, 1))
    assert relerr(Abar, orc.potrf_backward(Lh, w["Lbar"])) <= tol


@pytest.mark.parametrize("lengthscale,jitter", [(1.0, 1e-2), (3.0, 0.5)])
def test_c3_gp_marginal_likelihood(la, orc, lengthscale, jitter):
    # (1.0, 1e-2) is the configuration as stated (A is close to 1.01 I); (3.0, 0.5) has a dense
    # kernel matrix (cond <= 1e3) so the off-diagonal paths carry weight
    w = workloads.make("C3", lengthscale=lengthscale, jitter=jitter)
    tol = TOL[w["dtype"]]
    b, n = w["batch"], w["n"]
    assert np.all(workloads.cond_estimate(w["A"], sample=8) <= 1e3)
    A, y = dev(w["A"]), dev(w["y"])
    L = la.potrf(A)
    z = la.trsm(L, y.view(b, n, 1))
    alpha = la.trsm(L, z, trans=True)
    loss, Lbar = la.gp_glue(L, y, z.view(b, n), alpha.view(b, n))
    Abar = la.potrf_backward(L, Lbar)
    # oracle chain
    Lr = orc.potrf(w["A"])
    zr = orc.trsm(Lr, w["y"][..., None])
    ar = orc.trsm(Lr, zr, trans=True)
    loss_r, Lbar_r = orc.gp_glue(Lr, w["y"], zr[..., 0], ar[..., 0])
    Abar_r = orc.potrf_backward(Lr, Lbar_r)
    assert relerr(host(L), Lr) <= tol
    assert relerr(host(z), zr) <= tol
    assert relerr(host(alpha), ar) <= tol
    assert np.max(np.abs(host(loss) - loss_r) / np.maximum(np.abs(loss_r), 1.0)) <= tol
    assert relerr(host(Lbar), Lbar_r) <= tol
    assert relerr(host(Abar), Abar_r) <= tol
    # and the textbook gradient 1/2 (A^-1 - alpha alpha^T) as a second opinion on the whole chain
    Ai = np.linalg.inv(w["A"][:4].astype(np.float64))
    a = np.einsum("bij,bj->bi", Ai, w["y"][:4].astype(np.float64))
    assert relerr(host(Abar)[:4], 0.5 * (Ai - a[:, :, None] * a[:, None, :])) <= tol


def test_c4_medium_blocked(la, orc):
    w = workloads.make("C4")  # 32 matrices, n = 512, fp64, 64 right-hand sides
    tol = TOL[w["dtype"]]
    assert np.all(workloads.cond_estimate(w["A"], sample=2) <= 1e3)
    A, G, R = dev(w["A"]), dev(w["Lbar"]), dev(w["rhs"])
    L = la.potrf(A)
    X = la.trsm(L, R)
    Y = la.trmm(L, X)
    Abar = la.potrf_backward(L, G)
    Lr = orc.potrf(w["A"])
    Xr = orc.trsm(Lr, w["rhs"])
    assert relerr(host(L), Lr) <= tol
    assert relerr(host(X), Xr) <= tol
    assert relerr(host(Y), w["rhs"]) <= tol  # trmm undoes trsm
    assert relerr(host(Y), orc.trmm(Lr, Xr)) <= tol
    assert relerr(host(Abar), orc.potrf_backward(Lr, w["Lbar"])) <= tol


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_single_matrix_n1024_full_compare(la, orc, dtype):
    w = workloads.make("C5", n=1024, m=96, dtype=dtype)
    tol = TOL[dtype]
    A, G, R = dev(w["A"]), dev(w["Lbar"]), dev(w["rhs"])
    L = la.potrf(A)
    X = la.trsm(L, R)
    Abar = la.potrf_backward(L, G)
    Lr = orc.potrf(w["A"])
    assert relerr(host(L), Lr) <= tol
    assert relerr(host(X), orc.trsm(Lr, w["rhs"])) <= tol
    assert relerr(host(Abar), orc.potrf_backward(host(L), w["Lbar"])) <= tol


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_c5_large_single(la, orc, dtype):
    import torch

    w = workloads.make("C5", dtype=dtype)  # n = 8192, 512 right-hand sides
    n, m, tol = w["n"], w["m"], TOL[dtype]
    A_h, G_h, R_h = w["A"][0], w["Lbar"][0], w["rhs"][0]
    A, G, R = dev(w["A"]), dev(w["Lbar"]), dev(w["rhs"])
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    L = la.potrf(A, info=info)
    X = la.trsm(L, R)
    Abar = la.potrf_backward(L, G)
    half = la.potrf_backward(L, L.clone())  # closed form: Lbar = L  =>  Abar = I / 2
    Lh, Xh, Abar_h, half_h = host(L)[0], host(X)[0], host(Abar)[0], host(half)[0]
    assert int(host(info)[0]) == 0
    assert np.all(np.isfinite(Lh)) and np.all(np.isfinite(Abar_h))

    # (a) parts the oracle computes alone
    k = 768
    Lk = orc.potrf(A_h[:k, :k])
    assert relerr(Lh[:k, :k], Lk) <= tol
    assert relerr(Xh[:k], orc.trsm(Lk, R_h[:k])) <= tol
    assert np.all(np.triu(Lh, 1) == 0) and np.all(np.diag(Lh) > 0)

    # (b) sampled entries of the defining relations, each evaluated by the oracle
    rng = np.random.default_rng(8192)
    pts = [(0, 0), (n - 1, n - 1), (n - 1, 0), (n // 2, n // 2 - 1), (4095, 4096), (4096, 4095)]
    pts += [tuple(int(v) for v in rng.integers(0, n, size=2)) for _ in range(58)]
    L64 = Lh.astype(np.float64)
    scale_a = float(np.max(np.abs(A_h)))
    err_f = max(abs(orc.llt_entry(L64, i, j) - float(A_h[i, j])) for i, j in pts)
    sys.stderr.write(f"[c5 {dtype}] max |(L L^T - A)_ij| = {err_f:.3e} (scale {scale_a:.3e})\n")
    assert err_f <= tol * scale_a
    # sampled rows of L X = B (residual of the solve beyond the leading rows)
    rows = [n - 1, n // 2, 5000, 7001]
    resid = L64[rows] @ Xh.astype(np.float64) - R_h[rows]
    sys.stderr.write(f"[c5 {dtype}] max |(L X - B)_ij| = {np.max(np.abs(resid)):.3e} (scale {np.max(np.abs(R_h)):.3e})\n")
    assert np.max(np.abs(resid)) <= tol * float(np.max(np.abs(R_h)))
    # 2 L^T Abar L = copyltu(L^T Lbar) on sampled entries
    Ab64, G64 = Abar_h.astype(np.float64), G_h.astype(np.float64)
    worst, ref_scale = 0.0, 0.0
    for i, j in pts[:24]:
        lhs = 2.0 * orc.ltxl_entry(L64, Ab64, i, j)
        rhs = orc.ltlbar_entry(L64, G64, max(i, j), min(i, j))
        worst = max(worst, abs(lhs - rhs))
        ref_scale = max(ref_scale, abs(rhs))
    sys.stderr.write(f"[c5 {dtype}] max |(2 L^T Abar L - copyltu(L^T Lbar))_ij| = {worst:.3e} (scale {ref_scale:.3e})\n")
    assert worst <= tol * max(ref_scale, 1.0)
    assert np.array_equal(Abar_h, Abar_h.T)

    # (c) closed form through every tile
    assert relerr(half_h, 0.5 * np.eye(n)) <= tol
