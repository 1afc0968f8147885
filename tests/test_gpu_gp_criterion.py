"""Parity of la_gp_criterion (section 3.1: the Gaussian-process criterion and its gradient in
one call) against the oracle's chain potrf -> trsm -> trsm -> glue -> potrf backward on the
same seeded inputs, over sizes on both sides of the one-kernel limit, ragged sizes included."""
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


def rel(a, b):
    return float(np.linalg.norm(np.asarray(a, dtype=np.float64) - b) / max(np.linalg.norm(b), 1e-300))


def oracle_chain(orc, A, y):
    L = orc.potrf(A)
    z = orc.trsm(L, y[..., None])
    al = orc.trsm(L, z, trans=True)
    loss, Lbar = orc.gp_glue(L, y, z[..., 0], al[..., 0])
    return loss, orc.potrf_backward(L, Lbar)


def kernel_inputs(batch, n, dtype, lengthscale, jitter, seed):
    rng = np.random.default_rng(1000 * n + batch + seed)
    P = rng.uniform(-2.0, 2.0, size=(batch, n, 3))
    d2 = np.sum((P[:, :, None, :] - P[:, None, :, :]) ** 2, axis=-1)
    A = np.exp(-0.5 * d2 / lengthscale ** 2) + jitter * np.eye(n)
    y = rng.standard_normal((batch, n))
    dt = workloads.np_dtype(dtype)
    return A.astype(dt), y.astype(dt)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("batch,n", [(1, 1), (5, 2), (7, 15), (3, 16), (9, 17), (4, 33), (6, 64), (3, 80), (5, 96),
                                     (2, 97), (4, 128), (2, 129), (3, 200)])
def test_gp_criterion_parity(la, orc, dtype, batch, n):
    import torch

    A, y = kernel_inputs(batch, n, dtype, lengthscale=1.5, jitter=0.3, seed=0)
    assert np.linalg.cond(A[0].astype(np.float64)) <= 1e3
    loss_r, Abar_r = oracle_chain(orc, A, y)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    a, info = dev(A), torch.full((batch,), -1, dtype=torch.int32, device="cuda")
    loss, Abar = la.gp_criterion(a, dev(y), info=info)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert np.all(info.cpu().numpy() == 0)
    assert np.array_equal(a.cpu().numpy(), A)
    assert np.max(np.abs(loss.cpu().numpy() - loss_r) / np.maximum(np.abs(loss_r), 1.0)) <= tol
    got = Abar.cpu().numpy()
    assert np.array_equal(got, got.transpose(0, 2, 1))
    assert rel(got, Abar_r) <= tol
    # the gradient over A itself
    loss2, Abar2 = la.gp_criterion(a, dev(y), out=a)
    assert np.array_equal(Abar2.cpu().numpy(), got) and np.array_equal(loss2.cpu().numpy(), loss.cpu().numpy())


def test_gp_criterion_c3_and_second_opinion(la, orc):
    """The C3 configuration as stated and its dense-kernel variant; and the textbook gradient
    1/2 (A^-1 - alpha alpha^T) computed without any of the operators."""
    import torch

    for lengthscale, jitter in ((1.0, 1e-2), (3.0, 0.5)):
        w = workloads.make("C3", lengthscale=lengthscale, jitter=jitter)
        tol = TOL[w["dtype"]]
        loss_r, Abar_r = oracle_chain(orc, w["A"], w["y"])
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        loss, Abar = la.gp_criterion(dev(w["A"]), dev(w["y"]))
        assert np.max(np.abs(loss.cpu().numpy() - loss_r) / np.maximum(np.abs(loss_r), 1.0)) <= tol
        assert rel(Abar.cpu().numpy(), Abar_r) <= tol
        Ai = np.linalg.inv(w["A"][:4].astype(np.float64))
        al = np.einsum("bij,bj->bi", Ai, w["y"][:4].astype(np.float64))
        assert rel(Abar.cpu().numpy()[:4], 0.5 * (Ai - al[:, :, None] * al[:, None, :])) <= tol


def test_gp_criterion_reports_a_failing_pivot_and_bad_arguments(la):
    import ctypes

    import torch

    A, y = kernel_inputs(4, 40, "f64", 1.5, 0.3, seed=1)
    A[2] = -A[2]
    info = torch.full((4,), -1, dtype=torch.int32, device="cuda")
    la.gp_criterion(torch.from_numpy(A).cuda(), torch.from_numpy(y).cuda(), info=info)
    got = info.cpu().numpy()
    assert got[2] == 1 and np.all(np.delete(got, 2) == 0)
    lib = la.load()
    x = torch.zeros(300 * 300 * 2, dtype=torch.float64, device="cuda")
    p, z = ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(0)
    assert lib.la_gp_workspace_bytes(1, 2, 96) == 0 and lib.la_gp_workspace_bytes(0, 2, 128) == 0
    need = lib.la_gp_workspace_bytes(1, 2, 200)
    assert need >= (2 * 200 * 200 * 2 + 2 * 200 * 2) * 8  # L, Lbar, z, alpha, plus the scratch of the blocked operators
    q = ctypes.c_void_p(x.data_ptr() + 8 * 200 * 200 * 2)
    assert lib.la_gp_criterion(1, 2, 200, p, p, p, q, z, z, 0, z) == 4      # workspace missing (LA_ERR_WORKSPACE)
    assert lib.la_gp_criterion(1, 2, 40, p, p, z, q, z, z, 0, z) == 1       # no loss buffer
    assert lib.la_gp_criterion(5, 2, 40, p, p, p, q, z, z, 0, z) == 1       # bad dtype
    assert lib.la_gp_criterion(1, 0, 40, z, z, z, z, z, z, 0, z) == 0       # empty batch
